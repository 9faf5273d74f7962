// tree_pack and tree_accept: integer-only kernels, one 64-lane wavefront per
// sequence (trees hold at most 128 nodes, so a lane owns nodes lane, lane+64).
//
// The paper has the target model check a whole draft tree in one forward pass
// (Sec. 1) and keeps the prefix of a draft path the target agrees with (Sec. 3.1, below
// Eq. "cum_prob"); these kernels produce what that pass needs (positions,
// ancestor masks) and what it yields (the accepted path).
#include "common.h"

#include <cstring>

namespace {

constexpr int kWave = 64;

// The packing of one sequence by one wavefront; `parent_of(i)` yields the parent of local
// node i (from device memory, or from LDS when the tree was just fetched from the host).
template <typename ParentOf>
__device__ inline void pack_sequence(int b, int lane, int base, int n, int len, ParentOf parent_of,
                                     int32_t* __restrict__ depth, int32_t* __restrict__ position,
                                     int32_t* __restrict__ node_seq, uint64_t* __restrict__ anc_mask,
                                     int32_t* __restrict__ status) {
  bool ok = n >= 1 && n <= SMART_MAX_NODES;
  const int n_clamped = n < SMART_MAX_NODES ? n : SMART_MAX_NODES;
  // validate parents (lane-parallel), then agree across the wavefront
  bool mine_ok = true;
  for (int i = lane; i < n_clamped; i += kWave) {
    const int p = parent_of(i);
    mine_ok = mine_ok && (i == 0 ? p == -1 : (p >= 0 && p < i));
  }
  ok = ok && __all(mine_ok);
  for (int i = lane; i < n; i += kWave) {
    int d = 0;
    uint64_t lo = 0, hi = 0;
    if (ok) {
      // walk to the root; parent < child, so the walk is at most i steps
      for (int j = i; j >= 0; j = parent_of(j)) {
        if (j < 64) lo |= 1ull << j; else hi |= 1ull << (j - 64);
        ++d;
      }
      d -= 1;
    }
    depth[base + i] = d;
    position[base + i] = ok ? len + d : 0;
    node_seq[base + i] = ok ? b : 0;
    anc_mask[2 * (size_t)(base + i)] = lo;
    anc_mask[2 * (size_t)(base + i) + 1] = hi;
  }
  if (lane == 0) status[b] = ok ? SMART_OK : SMART_ETREE;
}

__global__ __launch_bounds__(kWave) void tree_pack_kernel(
    int batch, int total_nodes, const int32_t* __restrict__ cu_nodes,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ prefix_len,
    int32_t* __restrict__ depth, int32_t* __restrict__ position, int32_t* __restrict__ node_seq,
    uint64_t* __restrict__ anc_mask, int32_t* __restrict__ status) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  if (b >= batch) return;
  const int base = cu_nodes[b];
  const int end = cu_nodes[b + 1];
  // keep every access inside the arrays whatever the offsets say
  if (base < 0 || end < base || end > total_nodes) {
    if (lane == 0) status[b] = SMART_ETREE;
    return;
  }
  pack_sequence(b, lane, base, end - base, prefix_len[b], [&](int i) { return parent[base + i]; }, depth,
                position, node_seq, anc_mask, status);
}

// The offsets of a batch of at most 64 sequences travel in the kernel arguments (the host reads
// them from the pinned array when it launches), which saves the first of two round trips over
// the host link.
constexpr int kCuInArgs = 64;
struct CuArgs {
  int32_t v[kCuInArgs + 1];
};

// Small batches of small trees travel whole in the kernel arguments (the host copies parents and tokens out of
// the pinned arrays when it launches): no round trip over the host link is left in the kernel.
constexpr int kTreeInArgs = 448;  // nodes; with the offsets 3.9 KB of the 4 KB an argument block may have
struct TreeArgs {
  int32_t parent[kTreeInArgs];
  int32_t token[kTreeInArgs];
};
struct HostTrees {  // the trees where the caller left them: pinned host memory
  const int32_t* parent;
  const int32_t* token;
  __device__ int32_t parent_at(int i) const { return parent[i]; }
  __device__ int32_t token_at(int i) const { return token[i]; }
};
struct ArgTrees {  // the trees in the argument block
  const TreeArgs& t;
  __device__ int32_t parent_at(int i) const { return t.parent[i]; }
  __device__ int32_t token_at(int i) const { return t.token[i]; }
};

// tree_upload of the selected trees and tree_pack in one launch: the wavefront of sequence b
// fetches its tree (offsets, then nodes: from the arguments, or a round trip over the host link
// each), leaves device copies for the kernels that follow, and packs from LDS.
template <typename Trees>
__device__ inline void upload_pack_sequence(
    const CuArgs& cu_args, int cu_in_args, const Trees trees, bool with_tokens,
    int batch, int total_nodes, const int32_t* __restrict__ h_cu_nodes, int32_t* __restrict__ cu_nodes,
    int32_t* __restrict__ parent, int32_t* __restrict__ token, const int32_t* __restrict__ prefix_len,
    int32_t* __restrict__ depth, int32_t* __restrict__ position, int32_t* __restrict__ node_seq,
    uint64_t* __restrict__ anc_mask, int32_t* __restrict__ status, int32_t* par /* LDS, SMART_MAX_NODES */) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  if (b >= batch) return;
  const int base = cu_in_args ? cu_args.v[b] : h_cu_nodes[b];
  const int end = cu_in_args ? cu_args.v[b + 1] : h_cu_nodes[b + 1];
  const int len = prefix_len[b];
  if (lane == 0) {
    cu_nodes[b] = base;
    if (b == batch - 1) cu_nodes[batch] = end;
  }
  if (base < 0 || end < base || end > total_nodes) {
    if (lane == 0) status[b] = SMART_ETREE;
    return;
  }
  const int n = end - base;
  for (int i = lane; i < n; i += kWave) {
    const int p = trees.parent_at(base + i);
    parent[base + i] = p;
    if (i < SMART_MAX_NODES) par[i] = p;
    if (with_tokens) token[base + i] = trees.token_at(base + i);
  }
  __syncthreads();
  pack_sequence(b, lane, base, n, len, [&](int i) { return par[i]; }, depth, position, node_seq, anc_mask, status);
}

__global__ __launch_bounds__(kWave) void tree_upload_pack_kernel(
    const CuArgs cu_args, int cu_in_args,
    int batch, int total_nodes, const int32_t* __restrict__ h_cu_nodes, const int32_t* __restrict__ h_parent,
    const int32_t* __restrict__ h_token, int32_t* __restrict__ cu_nodes, int32_t* __restrict__ parent,
    int32_t* __restrict__ token, const int32_t* __restrict__ prefix_len, int32_t* __restrict__ depth,
    int32_t* __restrict__ position, int32_t* __restrict__ node_seq, uint64_t* __restrict__ anc_mask,
    int32_t* __restrict__ status) {
  __shared__ int32_t par[SMART_MAX_NODES];
  upload_pack_sequence(cu_args, cu_in_args, HostTrees{h_parent, h_token}, token != nullptr, batch, total_nodes,
                       h_cu_nodes, cu_nodes, parent, token, prefix_len, depth, position, node_seq, anc_mask, status,
                       par);
}

__global__ __launch_bounds__(kWave) void tree_upload_pack_args_kernel(
    const CuArgs cu_args, const TreeArgs tree_args, int with_tokens, int batch, int total_nodes,
    int32_t* __restrict__ cu_nodes, int32_t* __restrict__ parent, int32_t* __restrict__ token,
    const int32_t* __restrict__ prefix_len, int32_t* __restrict__ depth, int32_t* __restrict__ position,
    int32_t* __restrict__ node_seq, uint64_t* __restrict__ anc_mask, int32_t* __restrict__ status) {
  __shared__ int32_t par[SMART_MAX_NODES];
  // (total_nodes <= kTreeInArgs here, and the offsets are checked against total_nodes before anything is indexed)
  upload_pack_sequence(cu_args, 1, ArgTrees{tree_args}, with_tokens != 0, batch, total_nodes, nullptr, cu_nodes,
                       parent, token, prefix_len, depth, position, node_seq, anc_mask, status, par);
}

// The trees of a layer-at-a-time selection (`stride` entries per sequence, n[b] of them used)
// into CSR order, packed in the same launch.  Every wavefront sums the sizes before its own
// sequence itself: batches are small and this saves a scan kernel.
__global__ __launch_bounds__(kWave) void tree_compact_pack_kernel(
    int batch, int stride, const int32_t* __restrict__ n_of, const int32_t* __restrict__ s_parent,
    const int32_t* __restrict__ s_token, int32_t* __restrict__ cu_nodes, int32_t* __restrict__ parent,
    int32_t* __restrict__ token, const int32_t* __restrict__ prefix_len, int32_t* __restrict__ depth,
    int32_t* __restrict__ position, int32_t* __restrict__ node_seq, uint64_t* __restrict__ anc_mask,
    int32_t* __restrict__ status) {
  __shared__ int32_t par[SMART_MAX_NODES];
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  if (b >= batch) return;
  auto nodes_of = [&](int i) {
    const int n = n_of[i];
    return (n >= 1 && n <= stride) ? n : 0;
  };
  int before = 0;
  for (int i = lane; i < b; i += kWave) before += nodes_of(i);
  for (int sh = 32; sh >= 1; sh >>= 1) before += __shfl_xor(before, sh);
  const int base = before;
  const int n = nodes_of(b);
  if (lane == 0) {
    cu_nodes[b] = base;
    if (b == batch - 1) cu_nodes[batch] = base + n;
  }
  if (n == 0) {
    if (lane == 0) status[b] = SMART_ETREE;
    return;
  }
  for (int i = lane; i < n; i += kWave) {
    const int p = s_parent[(size_t)b * stride + i];
    parent[base + i] = p;
    par[i] = p;
    token[base + i] = s_token[(size_t)b * stride + i];
  }
  __syncthreads();
  pack_sequence(b, lane, base, n, prefix_len[b], [&](int i) { return par[i]; }, depth, position, node_seq,
                anc_mask, status);
}

__global__ __launch_bounds__(kWave) void tree_accept_kernel(
    int batch, int max_depth, const int32_t* __restrict__ cu_nodes,
    const int32_t* __restrict__ parent, const int32_t* __restrict__ token,
    const int32_t* __restrict__ target_next, int32_t* __restrict__ accept_len,
    int32_t* __restrict__ accept_path, int32_t* __restrict__ bonus_token) {
  const int b = blockIdx.x;
  const int lane = threadIdx.x;
  if (b >= batch) return;
  const int base = cu_nodes[b];
  const int n = cu_nodes[b + 1] - base;
  int32_t* path = accept_path + (size_t)b * (max_depth + 1);
  for (int d = lane; d <= max_depth; d += kWave) path[d] = -1;
  if (base < 0 || n < 1 || n > SMART_MAX_NODES) {
    if (lane == 0) { accept_len[b] = -1; bonus_token[b] = -1; }
    return;
  }
  // this lane's two nodes, and what the target puts after each (fetched with them: the walk below then needs no
  // further round trip, whatever its depth)
  const int i0 = lane, i1 = lane + kWave;
  const int p0 = i0 < n ? parent[base + i0] : -2, t0 = i0 < n ? token[base + i0] : 0;
  const int p1 = i1 < n ? parent[base + i1] : -2, t1 = i1 < n ? token[base + i1] : 0;
  const int next0 = i0 < n ? target_next[base + i0] : 0, next1 = i1 < n ? target_next[base + i1] : 0;
  auto target_after = [&](int node) {  // node is wave-uniform
    const int j = __builtin_amdgcn_readfirstlane(node);
    return j < kWave ? __builtin_amdgcn_readlane(next0, j) : __builtin_amdgcn_readlane(next1, j - kWave);
  };
  int cur = 0, len = 0;
  while (len < max_depth) {  // at most max_depth iterations, wave-uniform
    const int want = target_after(cur);
    const uint64_t m0 = __ballot(p0 == cur && t0 == want);
    const uint64_t m1 = __ballot(p1 == cur && t1 == want);
    int nxt;
    if (m0) nxt = __ffsll((unsigned long long)m0) - 1;
    else if (m1) nxt = kWave + __ffsll((unsigned long long)m1) - 1;
    else break;
    cur = nxt;
    ++len;
    if (lane == 0) path[len] = cur;
  }
  const int bonus = target_after(cur);
  if (lane == 0) {
    path[0] = 0;
    accept_len[b] = len;
    bonus_token[b] = bonus;
  }
}

// 16 bytes a lane where both sides are aligned, the ragged rest word by word.
__global__ __launch_bounds__(256) void tree_upload_kernel(const int32_t* __restrict__ src,
                                                          int32_t* __restrict__ dst, int64_t n_words,
                                                          int64_t n_vec) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n_vec) {
    reinterpret_cast<int4*>(dst)[i] = reinterpret_cast<const int4*>(src)[i];
  } else {
    const int64_t w = 4 * n_vec + (i - n_vec);
    if (w < n_words) dst[w] = src[w];
  }
}

}  // namespace

static bool device_can_address(const void* p) {
  hipPointerAttribute_t attr;
  if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return attr.type == hipMemoryTypeHost || attr.type == hipMemoryTypeDevice || attr.type == hipMemoryTypeManaged;
}

extern "C" int32_t tree_upload(smart_ctx* ctx, void* stream, const void* h_pinned_src, void* d_dst,
                               int64_t n_words) {
  if (!ctx || n_words < 0) return SMART_EINVAL;
  if (n_words == 0) return SMART_OK;
  if (!h_pinned_src || !d_dst) return SMART_EINVAL;
  // a kernel that dereferences pageable host memory faults: refuse what the device cannot address
  if (!device_can_address(h_pinned_src)) return SMART_EINVAL;
  const bool aligned = (reinterpret_cast<uintptr_t>(h_pinned_src) % 16 == 0) &&
                       (reinterpret_cast<uintptr_t>(d_dst) % 16 == 0);
  const int64_t n_vec = aligned ? n_words / 4 : 0;
  const int64_t threads = n_vec + (n_words - 4 * n_vec);
  const int64_t blocks = (threads + 255) / 256;
  if (blocks > 0x7fffffff) return SMART_EINVAL;
  hipLaunchKernelGGL(tree_upload_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                     static_cast<const int32_t*>(h_pinned_src), static_cast<int32_t*>(d_dst), n_words, n_vec);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t tree_upload_pack(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                                    const int32_t* h_pinned_cu_nodes, const int32_t* h_pinned_parent,
                                    const int32_t* h_pinned_token, int32_t* d_cu_nodes, int32_t* d_parent,
                                    int32_t* d_token, const int32_t* d_prefix_len, int32_t* d_depth,
                                    int32_t* d_position, int32_t* d_node_seq, uint64_t* d_anc_mask,
                                    int32_t* d_status) {
  if (!ctx || batch < 0 || total_nodes < 0) return SMART_EINVAL;
  if (!h_pinned_cu_nodes || !d_cu_nodes || !d_prefix_len || !d_status) return SMART_EINVAL;
  if ((h_pinned_token == nullptr) != (d_token == nullptr)) return SMART_EINVAL;
  if (total_nodes > 0 && (!h_pinned_parent || !d_parent || !d_depth || !d_position || !d_node_seq || !d_anc_mask))
    return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  // a kernel that dereferences pageable host memory faults: refuse what the device cannot address
  if (!device_can_address(h_pinned_cu_nodes) || (total_nodes > 0 && !device_can_address(h_pinned_parent)) ||
      (h_pinned_token && total_nodes > 0 && !device_can_address(h_pinned_token)))
    return SMART_EINVAL;
  // What travels in the arguments is what the pinned arrays hold NOW.  A launch that is being captured into a graph
  // runs later, perhaps many times, and must read the arrays when it runs: nothing travels then.
  // (the default stream cannot be captured, and asking about it while another stream is captured is an error)
  hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
  if (stream != nullptr && hipStreamIsCapturing((hipStream_t)stream, &capture) != hipSuccess) {
    (void)hipGetLastError();
    capture = hipStreamCaptureStatusNone;
  }
  CuArgs cu_args;
  const int cu_in_args = capture == hipStreamCaptureStatusNone && batch <= kCuInArgs;
  for (int b = 0; b <= kCuInArgs; ++b) cu_args.v[b] = cu_in_args && b <= batch ? h_pinned_cu_nodes[b] : 0;
  if (cu_in_args && total_nodes > 0 && total_nodes <= kTreeInArgs) {
    TreeArgs tree_args;
    std::memcpy(tree_args.parent, h_pinned_parent, sizeof(int32_t) * (size_t)total_nodes);
    if (h_pinned_token) std::memcpy(tree_args.token, h_pinned_token, sizeof(int32_t) * (size_t)total_nodes);
    hipLaunchKernelGGL(tree_upload_pack_args_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, cu_args,
                       tree_args, h_pinned_token ? 1 : 0, batch, total_nodes, d_cu_nodes, d_parent, d_token,
                       d_prefix_len, d_depth, d_position, d_node_seq, d_anc_mask, d_status);
    SMART_HIP_CHECK(hipGetLastError());
    return SMART_OK;
  }
  hipLaunchKernelGGL(tree_upload_pack_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, cu_args, cu_in_args,
                     batch, total_nodes, h_pinned_cu_nodes, h_pinned_parent, h_pinned_token, d_cu_nodes, d_parent,
                     d_token, d_prefix_len, d_depth, d_position, d_node_seq, d_anc_mask, d_status);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t tree_compact_pack(smart_ctx* ctx, void* stream, const smart_layer_state* d_state,
                                     int32_t total_cap, const int32_t* d_prefix_len, int32_t* d_cu_nodes,
                                     int32_t* d_parent, int32_t* d_token, int32_t* d_depth,
                                     int32_t* d_position, int32_t* d_node_seq, uint64_t* d_anc_mask,
                                     int32_t* d_status) {
  if (!ctx || !d_state || d_state->batch < 0 || d_state->budget < 1 || d_state->budget > SMART_MAX_NODES)
    return SMART_EINVAL;
  if (!d_cu_nodes || !d_prefix_len || !d_status) return SMART_EINVAL;
  const int32_t batch = d_state->batch;
  if (total_cap < 0 || (int64_t)total_cap < (int64_t)batch * d_state->budget) return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  if (!d_state->n || !d_state->parent || !d_state->token || !d_parent || !d_token || !d_depth || !d_position ||
      !d_node_seq || !d_anc_mask)
    return SMART_EINVAL;
  hipLaunchKernelGGL(tree_compact_pack_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, batch,
                     d_state->budget, d_state->n, d_state->parent, d_state->token, d_cu_nodes, d_parent, d_token,
                     d_prefix_len, d_depth, d_position, d_node_seq, d_anc_mask, d_status);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t tree_pack(smart_ctx* ctx, void* stream, int32_t batch, int32_t total_nodes,
                             const int32_t* d_cu_nodes, const int32_t* d_parent,
                             const int32_t* d_prefix_len, int32_t* d_depth, int32_t* d_position,
                             int32_t* d_node_seq, uint64_t* d_anc_mask, int32_t* d_status) {
  if (!ctx || batch < 0 || total_nodes < 0) return SMART_EINVAL;
  if (!d_cu_nodes || !d_prefix_len || !d_status) return SMART_EINVAL;
  if (total_nodes > 0 && (!d_parent || !d_depth || !d_position || !d_node_seq || !d_anc_mask))
    return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  hipLaunchKernelGGL(tree_pack_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, batch,
                     total_nodes, d_cu_nodes, d_parent, d_prefix_len, d_depth, d_position,
                     d_node_seq, d_anc_mask, d_status);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

extern "C" int32_t tree_accept(smart_ctx* ctx, void* stream, int32_t batch, int32_t max_depth,
                               const int32_t* d_cu_nodes, const int32_t* d_parent,
                               const int32_t* d_token, const int32_t* d_target_next,
                               int32_t* d_accept_len, int32_t* d_accept_path,
                               int32_t* d_bonus_token) {
  if (!ctx || batch < 0 || max_depth < 0 || max_depth > SMART_MAX_NODES) return SMART_EINVAL;
  if (!d_cu_nodes || !d_parent || !d_token || !d_target_next || !d_accept_len || !d_accept_path ||
      !d_bonus_token)
    return SMART_EINVAL;
  if (batch == 0) return SMART_OK;
  hipLaunchKernelGGL(tree_accept_kernel, dim3(batch), dim3(kWave), 0, (hipStream_t)stream, batch,
                     max_depth, d_cu_nodes, d_parent, d_token, d_target_next, d_accept_len,
                     d_accept_path, d_bonus_token);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}
