// tree_verify_attention, matrix-core path for bf16, head_dim 128, block_size 16,
// interleaved cache layout (gfx950 / CDNA4).
//
// The work splits in two, following where the bytes are:
//
//  * the cached prefix (thousands of keys per sequence, no mask) is a dense
//    contraction.  A 64-lane wavefront streams 32-key tiles of one
//    (sequence, kv head) and multiplies them against all rows of that kv head
//    at once -- rows = tree nodes x query heads of the GQA group -- so every
//    K/V byte leaves HBM once.  K and V vectors are loaded from HBM directly
//    in v_mfma_f32_32x32x16_bf16 operand layout (that is what the interleaved
//    cache layout is for), scores are kept transposed (keys x rows) so that a
//    row's softmax reduction stays inside a lane, and the probabilities come
//    out of the first product already in the operand layout of the second.
//    The key range of the whole batch is cut into equal shares, one per
//    wavefront ("worker"), independent of sequence boundaries, so ragged
//    prefix lengths do not unbalance the machine; each (worker, segment) pair
//    leaves an unnormalised partial (max, sum, O).
//
//  * the tree part (a node sees only itself and its ancestors: a handful of
//    keys selected by a 128-bit mask) is sparse and tiny.  It is evaluated in
//    fp32 on the vector ALUs inside the combine kernel, by walking the set
//    bits of the node's ancestor mask, and merged with the prefix partials by
//    the usual log-sum-exp merge.
//
// The paper (Sec. 1) only says that the tree is verified in one forward pass
// of the target model; this file is the attention sub-step of that pass.
#include <math.h>

#include "common.h"

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) float floatx8;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) float floatx4;
typedef __attribute__((ext_vector_type(4))) uint16_t ushortx4;
typedef __attribute__((ext_vector_type(8))) uint16_t ushortx8;

constexpr int kWave = 64;
constexpr int kD = 128;
constexpr int kBlock = 16;            // tokens per cache block
constexpr int kTile = 32;             // keys per tile = two cache blocks
constexpr int kRowsPerGroup = 64;     // query rows one worker carries (two 32-row MFMA tiles)
constexpr int kSlotFloats = kRowsPerGroup * kD + 2 * kRowsPerGroup;  // O, then max, then sum
constexpr int kCombineRows = 8;       // rows per combine wavefront (8 lanes per row)
constexpr int kMinTilesPerWorker = 8;
constexpr float kLog2e = 1.4426950408889634f;

// ---------------------------------------------------------------------------
// launch plan (device memory, written by tva_plan_kernel)
// ---------------------------------------------------------------------------
struct SeqInfo {
  int32_t len;    // prefix length, clamped
  int32_t n;      // tree nodes, clamped to [0, SMART_MAX_NODES]
  int32_t tiles;  // ceil(len / 32)
  int32_t rg;     // row groups = ceil(n * G / 64)
};

struct PlanView {
  int64_t* header;        // [0] total units U, [1] workers W
  int64_t* cum_units;     // [B+1] units before sequence b (unit = one tile of one (kv head, row group))
  int32_t* cum_segs;      // [B+1] segments before sequence b (segment = (kv head, row group))
  int32_t* cum_chunks;    // [B+1] combine row chunks before sequence b
  SeqInfo* info;          // [B]
};

__host__ __device__ inline size_t plan_bytes_for(int batch) {
  return sizeof(int64_t) * (8 + (size_t)batch + 1) + sizeof(int32_t) * 2 * ((size_t)batch + 2) +
         sizeof(SeqInfo) * (size_t)batch + 64;
}

__host__ __device__ inline PlanView plan_view(void* base, int batch) {
  PlanView v;
  char* p = (char*)base;
  v.header = (int64_t*)p;
  p += sizeof(int64_t) * 8;
  v.cum_units = (int64_t*)p;
  p += sizeof(int64_t) * ((size_t)batch + 1);
  v.info = (SeqInfo*)p;
  p += sizeof(SeqInfo) * (size_t)batch;
  v.cum_segs = (int32_t*)p;
  p += sizeof(int32_t) * ((size_t)batch + 2);
  v.cum_chunks = (int32_t*)p;
  return v;
}

// One workgroup.  Thread t owns a contiguous range of sequences; a serial scan
// over the per-thread sums (256 entries) ties the ranges together.
__global__ __launch_bounds__(256) void tva_plan_kernel(
    void* plan_base, int batch, int total_nodes, int G, int Hkv, int max_blocks, int max_workers,
    const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ cu_nodes) {
  __shared__ int64_t s_units[256];
  __shared__ int32_t s_segs[256], s_chunks[256];
  PlanView pv = plan_view(plan_base, batch);
  const int t = threadIdx.x;
  const int per = (batch + 255) / 256;
  const int b0 = t * per, b1 = min(batch, b0 + per);
  int64_t units = 0;
  int32_t segs = 0, chunks = 0;
  for (int b = b0; b < b1; ++b) {
    int len = prefix_len[b];
    const int cap = max_blocks * kBlock;
    len = len < 0 ? 0 : (len > cap ? cap : len);
    const int base = cu_nodes[b];
    int n = cu_nodes[b + 1] - base;
    if (base < 0 || n < 0 || base + n > total_nodes) n = 0;
    n = n > SMART_MAX_NODES ? SMART_MAX_NODES : n;
    SeqInfo si;
    si.len = len;
    si.n = n;
    si.tiles = (len + kTile - 1) / kTile;
    si.rg = (n * G + kRowsPerGroup - 1) / kRowsPerGroup;
    pv.info[b] = si;
    units += (int64_t)si.tiles * Hkv * si.rg;
    segs += Hkv * si.rg;
    chunks += Hkv * ((n * G + kCombineRows - 1) / kCombineRows);
  }
  s_units[t] = units;
  s_segs[t] = segs;
  s_chunks[t] = chunks;
  __syncthreads();
  if (t == 0) {
    int64_t u = 0;
    int32_t s = 0, c = 0;
    for (int i = 0; i < 256; ++i) {
      const int64_t uu = s_units[i];
      const int32_t ss = s_segs[i], cc = s_chunks[i];
      s_units[i] = u; s_segs[i] = s; s_chunks[i] = c;
      u += uu; s += ss; c += cc;
    }
    pv.cum_units[batch] = u;
    pv.cum_segs[batch] = s;
    pv.cum_chunks[batch] = c;
    int64_t w = u / kMinTilesPerWorker;
    w = w < 1 ? 1 : (w > max_workers ? max_workers : w);
    pv.header[0] = u;
    pv.header[1] = w;
  }
  __syncthreads();
  units = s_units[t];
  segs = s_segs[t];
  chunks = s_chunks[t];
  for (int b = b0; b < b1; ++b) {
    const SeqInfo si = pv.info[b];
    pv.cum_units[b] = units;
    pv.cum_segs[b] = segs;
    pv.cum_chunks[b] = chunks;
    units += (int64_t)si.tiles * Hkv * si.rg;
    segs += Hkv * si.rg;
    chunks += Hkv * ((si.n * G + kCombineRows - 1) / kCombineRows);
  }
}

// ---------------------------------------------------------------------------
// prefix kernel
// ---------------------------------------------------------------------------
struct MainArgs {
  const __bf16* q;
  const __bf16* k_cache;
  const __bf16* v_cache;
  const int32_t* block_table;
  const int32_t* cu_nodes;
  void* plan;
  float* ws;
  int64_t block_stride, head_stride;
  int32_t batch, Hq, Hkv, G, max_blocks, num_blocks;
  float scale_log2e;
};

// Row m of a 16-row half of the score tile holds cache slot sigma(m): swapping
// bits 2 and 3 makes the 8 accumulator registers a lane ends up with (rows
// 4h..4h+3 and 8+4h..8+4h+3 of each half) cover 8 consecutive slots, which is
// one V vector of the interleaved layout.
__device__ inline int sigma(int m) { return (m & 3) | ((m & 4) << 1) | ((m & 8) >> 1); }

struct KVTile {
  bf16x8 k[8];     // A operand of scores: [k step]
  bf16x8 v[2][4];  // A operand of the output product: [cache block of the tile][32-wide d tile]
};

__device__ inline void load_tile(KVTile& T, const MainArgs& a, const int32_t* bt_row, int tile,
                                 int n_blocks, int g, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const int i0 = 2 * tile;
  const int i1 = min(2 * tile + 1, n_blocks - 1);  // a missing second block is fully masked later
  int64_t blk0 = bt_row[i0], blk1 = bt_row[i1];
  blk0 = blk0 < 0 ? 0 : (blk0 >= a.num_blocks ? a.num_blocks - 1 : blk0);
  blk1 = blk1 < 0 ? 0 : (blk1 >= a.num_blocks ? a.num_blocks - 1 : blk1);
  const int64_t page0 = blk0 * a.block_stride + (int64_t)g * a.head_stride;
  const int64_t page1 = blk1 * a.block_stride + (int64_t)g * a.head_stride;
  const __bf16* kp = a.k_cache + ((j >> 4) ? page1 : page0) + (h * 16 + sigma(j & 15)) * 8;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) T.k[ks] = *(const bf16x8*)(kp + ks * 256);
  const __bf16* vp0 = a.v_cache + page0 + (h * kD + j) * 8;
  const __bf16* vp1 = a.v_cache + page1 + (h * kD + j) * 8;
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    T.v[0][jt] = *(const bf16x8*)(vp0 + jt * 256);
    T.v[1][jt] = *(const bf16x8*)(vp1 + jt * 256);
  }
}

template <int QT>
struct RowState {
  bf16x8 q[QT][8];     // B operand of scores
  floatx16 o[QT][4];   // output accumulators, transposed: [d tile], lane = query row
  float m[QT], l[QT];  // running max (raw score units) and this lane's share of the sum
};

template <int QT>
__device__ inline void compute_tile(RowState<QT>& R, KVTile& T, int n_valid, float c, int lane) {
  const int h = lane >> 5;
  floatx16 s[QT];
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    s[qt] = (floatx16)(0.f);
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      s[qt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(T.k[ks], R.q[qt][ks], s[qt], 0, 0, 0);
  }
  if (n_valid < kTile) {  // ragged end of the prefix (wave-uniform)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int i = 8 * (r >> 2) + 4 * h + (r & 3);     // score-tile row of this register
      const int tok = (i & 16) + sigma(i & 15);         // token of the tile it holds
      if (tok >= n_valid) {
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) s[qt][r] = -INFINITY;
      }
    }
    // unused cache slots may hold anything, NaN included: zero them in V
#pragma unroll
    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (kk * 16 + h * 8 + e >= n_valid) {
#pragma unroll
          for (int jt = 0; jt < 4; ++jt) T.v[kk][jt][e] = (__bf16)0.f;
        }
  }
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    float mx = s[qt][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[qt][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(R.m[qt], mx);
    if (__any(m_new > R.m[qt])) {  // rescale only when some row's maximum moved
      const float alpha = __builtin_amdgcn_exp2f((R.m[qt] - m_new) * c);
      R.l[qt] *= alpha;
#pragma unroll
      for (int jt = 0; jt < 4; ++jt) R.o[qt][jt] *= alpha;
      R.m[qt] = m_new;
    }
    const float mc = R.m[qt] * c;
    floatx8 p0, p1;
    float sum = 0.f;
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      p0[r] = __builtin_amdgcn_exp2f(fmaf(s[qt][r], c, -mc));
      p1[r] = __builtin_amdgcn_exp2f(fmaf(s[qt][r + 8], c, -mc));
      sum += p0[r] + p1[r];
    }
    R.l[qt] += sum;
    const bf16x8 pb0 = __builtin_convertvector(p0, bf16x8);
    const bf16x8 pb1 = __builtin_convertvector(p1, bf16x8);
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
      R.o[qt][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(T.v[0][jt], pb0, R.o[qt][jt], 0, 0, 0);
      R.o[qt][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(T.v[1][jt], pb1, R.o[qt][jt], 0, 0, 0);
    }
  }
}

// Streams tiles [t0, t1) of (sequence b, kv head g) against row group `rgi`
// and writes the unnormalised partial to `slot`.
template <int QT>
__device__ inline void process_segment(const MainArgs& a, int b, int g, int rgi, int t0, int t1,
                                       const SeqInfo si, float* slot, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const int M = si.n * a.G;
  const int base = a.cu_nodes[b];
  RowState<QT> R;
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    int rho = rgi * kRowsPerGroup + qt * 32 + j;
    rho = rho < M ? rho : M - 1;  // padding rows repeat the last real row; never read back
    const int node = base + rho / a.G, head = g * a.G + rho % a.G;
    const __bf16* qp = a.q + ((int64_t)node * a.Hq + head) * kD + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) R.q[qt][ks] = *(const bf16x8*)(qp + ks * 16);
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) R.o[qt][jt] = (floatx16)(0.f);
    R.m[qt] = -INFINITY;
    R.l[qt] = 0.f;
  }
  const int32_t* bt_row = a.block_table + (int64_t)b * a.max_blocks;
  const int n_blocks = (si.len + kBlock - 1) / kBlock;
  const float c = a.scale_log2e;

  KVTile A, B;
  load_tile(A, a, bt_row, t0, n_blocks, g, lane);
  int t = t0;
  while (t + 1 < t1) {
    load_tile(B, a, bt_row, t + 1, n_blocks, g, lane);
    compute_tile<QT>(R, A, min(kTile, si.len - t * kTile), c, lane);
    if (t + 2 < t1) load_tile(A, a, bt_row, t + 2, n_blocks, g, lane);
    compute_tile<QT>(R, B, min(kTile, si.len - (t + 1) * kTile), c, lane);
    t += 2;
  }
  if (t < t1) compute_tile<QT>(R, A, min(kTile, si.len - t * kTile), c, lane);

  // partial: O as [row tile][d / 4][row][4] so that lanes write contiguous 16-byte pieces
#pragma unroll
  for (int qt = 0; qt < QT; ++qt) {
    const float l = R.l[qt] + __shfl_xor(R.l[qt], 32);
#pragma unroll
    for (int jt = 0; jt < 4; ++jt)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        const int chunk = jt * 8 + 2 * r4 + h;
        floatx4 v;
        v[0] = R.o[qt][jt][4 * r4 + 0];
        v[1] = R.o[qt][jt][4 * r4 + 1];
        v[2] = R.o[qt][jt][4 * r4 + 2];
        v[3] = R.o[qt][jt][4 * r4 + 3];
        *(floatx4*)(slot + ((size_t)(qt * 32 + chunk) * 32 + j) * 4) = v;
      }
    if (h == 0) {
      slot[kRowsPerGroup * kD + qt * 32 + j] = R.m[qt];
      slot[kRowsPerGroup * kD + kRowsPerGroup + qt * 32 + j] = l;
    }
  }
}

// One wavefront per worker.  Worker w owns units [w U / W, (w+1) U / W) of the
// batch-wide sequence of (sequence, kv head, row group, tile) units.
__global__ __launch_bounds__(kWave) void tva_prefix_kernel(MainArgs a) {
  const PlanView pv = plan_view(a.plan, a.batch);
  const int64_t U = pv.header[0], W = pv.header[1];
  const int64_t w = blockIdx.x;
  if (w >= W || U <= 0) return;
  int64_t u0 = (w * U) / W;
  const int64_t u1 = ((w + 1) * U) / W;
  if (u0 >= u1) return;
  const int lane = threadIdx.x;
  // sequence that holds unit u0: last b with cum_units[b] <= u0
  int lo = 0, hi = a.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (pv.cum_units[mid] <= u0) lo = mid; else hi = mid;
  }
  int b = lo;
  while (u0 < u1 && b < a.batch) {
    const SeqInfo si = pv.info[b];
    const int64_t seq_begin = pv.cum_units[b], seq_end = pv.cum_units[b + 1];
    if (u0 >= seq_end) { ++b; continue; }  // also skips sequences without units
    const int64_t local = u0 - seq_begin;
    const int seg_local = (int)(local / si.tiles);
    const int t0 = (int)(local % si.tiles);
    const int g = seg_local / si.rg, rgi = seg_local % si.rg;
    const int64_t left = u1 - u0;
    const int nt = (int)(left < (int64_t)(si.tiles - t0) ? left : (int64_t)(si.tiles - t0));
    const int64_t seg = (int64_t)pv.cum_segs[b] + seg_local;
    float* slot = a.ws + (size_t)(w + seg) * kSlotFloats;
    const int rows = si.n * a.G - rgi * kRowsPerGroup;
    if (rows > 32) process_segment<2>(a, b, g, rgi, t0, t0 + nt, si, slot, lane);
    else process_segment<1>(a, b, g, rgi, t0, t0 + nt, si, slot, lane);
    u0 += nt;
  }
}

// ---------------------------------------------------------------------------
// combine kernel: tree part on the vector ALUs + merge of the prefix partials
// ---------------------------------------------------------------------------
struct CombineArgs {
  const uint16_t* q;
  const uint16_t* k_tree;
  const uint16_t* v_tree;
  const int32_t* cu_nodes;
  const uint64_t* anc_mask;
  void* plan;
  const float* ws;
  uint16_t* out;
  float* lse;
  int32_t batch, Hq, Hkv, G;
  float scale, scale_log2e;
};

__device__ inline float bf16_to_f32(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
__device__ inline uint16_t f32_to_bf16(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// 8 lanes per query row; lane e of a row owns d = 4c .. 4c+3 for c = e, e+8, e+16, e+24.
__global__ __launch_bounds__(kWave) void tva_combine_kernel(CombineArgs a) {
  const PlanView pv = plan_view(a.plan, a.batch);
  const int wc = blockIdx.x;
  if (wc >= pv.cum_chunks[a.batch]) return;
  int lo = 0, hi = a.batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (pv.cum_chunks[mid] <= wc) lo = mid; else hi = mid;
  }
  const int b = lo;
  const SeqInfo si = pv.info[b];
  const int M = si.n * a.G;
  const int per_g = (M + kCombineRows - 1) / kCombineRows;
  const int local = wc - pv.cum_chunks[b];
  const int g = local / per_g, chunk = local % per_g;
  const int lane = threadIdx.x;
  const int e = lane & 7;
  const int rho_raw = chunk * kCombineRows + (lane >> 3);
  const bool active = rho_raw < M;
  const int rho = active ? rho_raw : M - 1;
  const int base = a.cu_nodes[b];
  const int node = base + rho / a.G, head = g * a.G + rho % a.G;
  const float c = a.scale_log2e;

  float qv[16];
  {
    const uint16_t* qp = a.q + ((int64_t)node * a.Hq + head) * kD;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const ushortx4 x = *(const ushortx4*)(qp + 4 * (e + 8 * k));
#pragma unroll
      for (int i = 0; i < 4; ++i) qv[4 * k + i] = bf16_to_f32(x[i]);
    }
  }
  float m = -INFINITY, l = 0.f, acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  // tree keys: the set bits of this row's ancestor mask, lowest first
  uint64_t mlo = active ? a.anc_mask[2 * (size_t)node] : 0ull;
  uint64_t mhi = active ? a.anc_mask[2 * (size_t)node + 1] : 0ull;
  if (si.n < 64) mlo &= (1ull << si.n) - 1ull, mhi = 0ull;           // never index past the tree
  else if (si.n < 128) mhi &= (1ull << (si.n - 64)) - 1ull;
  while (__any((mlo | mhi) != 0ull)) {
    const bool have = (mlo | mhi) != 0ull;
    int jn = 0;
    if (mlo) { jn = __ffsll((unsigned long long)mlo) - 1; mlo &= mlo - 1; }
    else if (mhi) { jn = 64 + __ffsll((unsigned long long)mhi) - 1; mhi &= mhi - 1; }
    const uint16_t* kp = a.k_tree + ((int64_t)(base + jn) * a.Hkv + g) * kD;
    const uint16_t* vp = a.v_tree + ((int64_t)(base + jn) * a.Hkv + g) * kD;
    float dot = 0.f;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const ushortx4 x = *(const ushortx4*)(kp + 4 * (e + 8 * k));
#pragma unroll
      for (int i = 0; i < 4; ++i) dot = fmaf(qv[4 * k + i], bf16_to_f32(x[i]), dot);
    }
    dot += __shfl_xor(dot, 1);
    dot += __shfl_xor(dot, 2);
    dot += __shfl_xor(dot, 4);
    if (have) {
      const float m_new = fmaxf(m, dot);
      const float al = __builtin_amdgcn_exp2f((m - m_new) * c);
      const float p = __builtin_amdgcn_exp2f((dot - m_new) * c);
      l = l * al + p;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const ushortx4 x = *(const ushortx4*)(vp + 4 * (e + 8 * k));
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[4 * k + i] = acc[4 * k + i] * al + p * bf16_to_f32(x[i]);
      }
      m = m_new;
    }
  }

  // prefix partials of this row's segment: workers w_first .. w_last
  if (si.tiles > 0 && active) {
    const int64_t U = pv.header[0], W = pv.header[1];
    const int rgi = rho / kRowsPerGroup;
    const int seg_local = g * si.rg + rgi;
    const int64_t seg = (int64_t)pv.cum_segs[b] + seg_local;
    const int64_t ub = pv.cum_units[b] + (int64_t)seg_local * si.tiles;
    const int64_t ue = ub + si.tiles - 1;
    const int64_t w_first = ((ub + 1) * W - 1) / U;
    const int64_t w_last = ((ue + 1) * W - 1) / U;
    const int row = rho % kRowsPerGroup;  // = qt * 32 + j
    const int qt = row >> 5, j = row & 31;
    for (int64_t w = w_first; w <= w_last; ++w) {
      const float* slot = a.ws + (size_t)(w + seg) * kSlotFloats;
      const float mc = slot[kRowsPerGroup * kD + row];
      const float lc = slot[kRowsPerGroup * kD + kRowsPerGroup + row];
      const float m_new = fmaxf(m, mc);
      const float al = __builtin_amdgcn_exp2f((m - m_new) * c);
      const float wt = __builtin_amdgcn_exp2f((mc - m_new) * c);
      l = l * al + lc * wt;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const floatx4 x = *(const floatx4*)(slot + ((size_t)(qt * 32 + e + 8 * k) * 32 + j) * 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[4 * k + i] = acc[4 * k + i] * al + wt * x[i];
      }
      m = m_new;
    }
  }
  if (!active) return;
  const float inv = l > 0.f ? 1.f / l : 0.f;
  uint16_t* op = a.out + ((int64_t)node * a.Hq + head) * kD;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    ushortx4 y;
#pragma unroll
    for (int i = 0; i < 4; ++i) y[i] = f32_to_bf16(acc[4 * k + i] * inv);
    *(ushortx4*)(op + 4 * (e + 8 * k)) = y;
  }
  if (a.lse && e == 0)
    a.lse[(int64_t)node * a.Hq + head] = l > 0.f ? m * a.scale + logf(l) : -INFINITY;
}

}  // namespace

namespace smart {

int32_t tva_mfma_default_workers(const smart_ctx* ctx) {
  // one wavefront per SIMD: 4 per compute unit
  return (ctx->num_cus > 0 ? ctx->num_cus : 256) * 4;
}

void tva_mfma_workspace(int32_t batch, int32_t total_nodes, int32_t num_q_heads,
                        int32_t num_kv_heads, int32_t workers, size_t* ws_bytes,
                        size_t* plan_bytes) {
  const int64_t G = num_q_heads / num_kv_heads;
  const int64_t segs = (int64_t)num_kv_heads * (((int64_t)total_nodes * G + kRowsPerGroup - 1) / kRowsPerGroup + batch);
  const int64_t slots = (int64_t)workers + segs + 1;
  *ws_bytes = (size_t)slots * kSlotFloats * sizeof(float);
  *plan_bytes = plan_bytes_for(batch);
}

bool tva_mfma_supported(const tva_params& p) {
  auto aligned16 = [](const void* x) { return ((uintptr_t)x & 15u) == 0; };
  return p.dtype == SMART_BF16 && p.kv_layout == SMART_KV_INTERLEAVED && p.head_dim == kD &&
         p.block_size == kBlock && p.cache_block_stride % 8 == 0 && p.cache_head_stride % 8 == 0 &&
         aligned16(p.d_q) && aligned16(p.d_k_cache) && aligned16(p.d_v_cache) &&
         aligned16(p.d_k_tree) && aligned16(p.d_v_tree) && aligned16(p.d_out) && p.num_blocks > 0;
}

int32_t tva_launch_mfma(smart_ctx* ctx, hipStream_t stream, const tva_params& p) {
  if (p.batch == 0 || p.total_nodes == 0) return SMART_OK;
  const int G = p.num_q_heads / p.num_kv_heads;
  const int32_t workers = ctx->opt_workers > 0 ? (int32_t)ctx->opt_workers : tva_mfma_default_workers(ctx);
  size_t ws_bytes = 0, plan_bytes = 0;
  tva_mfma_workspace(p.batch, p.total_nodes, p.num_q_heads, p.num_kv_heads, workers, &ws_bytes, &plan_bytes);
  int32_t rc = ensure_workspace(ctx, stream, ws_bytes, plan_bytes);
  if (rc != SMART_OK) return rc;

  hipLaunchKernelGGL(tva_plan_kernel, dim3(1), dim3(256), 0, stream, (void*)ctx->plan, p.batch,
                     p.total_nodes, G, p.num_kv_heads, p.max_blocks_per_seq, workers,
                     p.d_prefix_len, p.d_cu_nodes);
  SMART_HIP_CHECK(hipGetLastError());

  MainArgs ma;
  ma.q = (const __bf16*)p.d_q;
  ma.k_cache = (const __bf16*)p.d_k_cache;
  ma.v_cache = (const __bf16*)p.d_v_cache;
  ma.block_table = p.d_block_table;
  ma.cu_nodes = p.d_cu_nodes;
  ma.plan = ctx->plan;
  ma.ws = (float*)ctx->ws;
  ma.block_stride = p.cache_block_stride;
  ma.head_stride = p.cache_head_stride;
  ma.batch = p.batch;
  ma.Hq = p.num_q_heads;
  ma.Hkv = p.num_kv_heads;
  ma.G = G;
  ma.max_blocks = p.max_blocks_per_seq;
  ma.num_blocks = p.num_blocks;
  ma.scale_log2e = p.softmax_scale * kLog2e;
  hipLaunchKernelGGL(tva_prefix_kernel, dim3(workers), dim3(kWave), 0, stream, ma);
  SMART_HIP_CHECK(hipGetLastError());

  CombineArgs ca;
  ca.q = (const uint16_t*)p.d_q;
  ca.k_tree = (const uint16_t*)p.d_k_tree;
  ca.v_tree = (const uint16_t*)p.d_v_tree;
  ca.cu_nodes = p.d_cu_nodes;
  ca.anc_mask = p.d_anc_mask;
  ca.plan = ctx->plan;
  ca.ws = (const float*)ctx->ws;
  ca.out = (uint16_t*)p.d_out;
  ca.lse = p.d_lse;
  ca.batch = p.batch;
  ca.Hq = p.num_q_heads;
  ca.Hkv = p.num_kv_heads;
  ca.G = G;
  ca.scale = p.softmax_scale;
  ca.scale_log2e = p.softmax_scale * kLog2e;
  const int64_t max_chunks =
      (int64_t)p.num_kv_heads * (((int64_t)p.total_nodes * G + kCombineRows - 1) / kCombineRows + p.batch);
  if (max_chunks > 0x7FFFFFFF) return SMART_EINVAL;
  hipLaunchKernelGGL(tva_combine_kernel, dim3((unsigned)max_chunks), dim3(kWave), 0, stream, ca);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

}  // namespace smart
