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
//    worker, independent of sequence boundaries, so ragged prefix lengths do
//    not unbalance the machine; each (worker, segment) pair leaves an
//    unnormalised partial (max, sum, O).  Sequences fall in three classes by
//    their rows per kv head (<= 32, <= 64, more); ONE kernel launch serves all
//    three, its workgroups dealt to the classes in proportion to their work:
//    class 0 streams K/V from HBM straight into operand registers (eight
//    wavefronts share a worker's tiles); classes 1 and 2 stage tiles in LDS
//    (HBM -> LDS without passing through registers) for the eight wavefronts
//    of a workgroup: two row tiles x two key groups in class 1, eight row
//    tiles of 32 rows each in class 2.
//
//  * the tree part (a node sees only itself and its ancestors: a handful of
//    keys selected by a 128-bit mask) is sparse and tiny.  It is evaluated in
//    fp32 on the vector ALUs inside the combine kernel, by walking the set
//    bits of the node's ancestor mask, and merged with the prefix partials by
//    the usual log-sum-exp merge.
//
// The paper (Sec. 1) only says that the tree is verified in one forward pass
// of the target model; this file is the attention sub-step of that pass.
#include <hip/hip_ext.h>
#include <math.h>

#include "common.h"

// The timeline build (-DSMART_TVA_TIMELINE, a library of its own: libsmart_tree_timeline.so, read by
// python -m paper_2604_09731_amd.timeline) keeps wall-clock stamps (100 MHz counter) of the LAST launch: per
// workgroup of the prefix kernel its start, end, shader cycles and class; per wavefront of the combine kernel its
// start and end.  Nothing of this is in the ordinary library.
#ifdef SMART_TVA_TIMELINE
namespace timeline {
constexpr int kWorkgroups = 1024, kWaves = 16384;
__device__ unsigned long long wg_stamps[kWorkgroups * 4];  // start, end, shader cycles, class | worker << 8
__device__ unsigned long long wave_stamps[kWaves * 2];     // start, end
}  // namespace timeline
#define SMART_TIMELINE(...) __VA_ARGS__
#else
#define SMART_TIMELINE(...)
#endif

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
constexpr int kClasses = 3;           // sequences are classed by rows = nodes x group heads per kv head
constexpr int kSmallRows = 32;        // class 0: all rows fit one 32-row MFMA tile
constexpr int kMediumRows = 64;       // class 1: all rows fit two 32-row MFMA tiles
constexpr int kLargeRows = 256;       // class 2: row groups of 256 = one workgroup of eight wavefronts x 32 rows
constexpr int kWgWaves = 8;           // wavefronts per workgroup of the prefix kernel (two per SIMD)
constexpr int kSmallSlot = kSmallRows * kD + 2 * kSmallRows;  // floats: O, then max, then sum
constexpr int kMediumSlot = kMediumRows * kD + 2 * kMediumRows;
constexpr int kLargeSlot = kLargeRows * kD + 2 * kLargeRows;
__host__ __device__ inline int class_rows(int cls) { return cls == 0 ? kSmallRows : (cls == 1 ? kMediumRows : kLargeRows); }
__host__ __device__ inline int class_slot(int cls) { return cls == 0 ? kSmallSlot : (cls == 1 ? kMediumSlot : kLargeSlot); }
constexpr int kCombineRows = 8;       // rows per combine wavefront (8 lanes per row)
constexpr int kMinTilesPerWorker[kClasses] = {16, 16, 8};  // workers are 8-wave workgroups
constexpr int kChunkTiles = 64;       // tiles whose block ids one pair of registers holds
constexpr float kLog2e = 1.4426950408889634f;
// Online softmax with a lazy reference: the value m that the exponentials are taken against follows the running
// maximum only when the maximum has moved more than 2^kRescaleStep above it (in the exponent's units), so the
// accumulators are rescaled a few times per segment instead of on most tiles; until then probabilities may reach
// 2^kRescaleStep instead of 1, which binary32 sums and bf16 operands carry at the same relative precision.  The
// partial's (m, l, O) stay consistent with each other, which is all the merges downstream need.
constexpr float kRescaleStep = 8.f;
// Every K/V byte of the cache is read once per call: the loads are marked nontemporal (streaming), which on this
// machine lifts a plain read stream from about 6.1 to 7.0 TB/s.  The same hint as a cache-policy operand (the nt
// bit) for the loads that go straight to LDS.
constexpr int kStreamPolicy = 2;

// ---------------------------------------------------------------------------
// launch plan (device memory; written by tva_plan_kernel, or for batches of at most 64
// sequences by workgroup 0 of the prefix kernel)
//
// A "unit" is one 32-key tile of one (sequence, kv head, row group) segment.
// Sequences fall in three classes with separate unit spaces:
//   class 0  n * G <= 32 rows: one row group, eight wavefronts share a worker's tiles
//   class 1  33 .. 64 rows: one row group, tiles staged in LDS, two key groups of wavefronts
//   class 2  more rows: row groups of 256 rows, eight wavefronts x 32 rows per worker
// ---------------------------------------------------------------------------
struct SeqInfo {
  int32_t len;    // prefix length, clamped
  int32_t n;      // tree nodes, clamped to [0, SMART_MAX_NODES]
  int32_t tiles;  // ceil(len / 32)
  int32_t rg;     // row groups (1 for class 1)
};

// Class 2 shares its workers by time rather than by tiles.  The eight wavefronts of a workgroup take one 32-row
// tile each (two per SIMD), so a 32-key tile of a segment with up to four row tiles takes what one wavefront
// takes (measured: 0.68 .. 0.76 us), and with five or more what two on one SIMD take (0.9 .. 1.07 us).  In units
// of 0.06 us: kLargeTileCost[row tiles] per tile.  (Starting and finishing a piece takes 11 .. 13 us on top; a
// start cost per segment in the unit space, 0 .. 200 units, changed nothing measurable and is not modelled.)
constexpr int kLargeTileCost[kLargeRows / 32 + 1] = {11, 11, 11, 12, 12, 16, 16, 17, 17};
// (the same currency for a tile of classes 0 and 1, for dealing the workgroups to the classes)
constexpr int kClassTileCost[kClasses] = {10, 10, 1};
constexpr int kFp8StreamTileCost = 5;

// What the unit space of class 2 holds of one sequence: per kv head its row groups in order, all but the last
// with eight row tiles.
struct LargeSpans {
  int32_t cost_last;   // cost of a tile of the last row group
  int64_t span_full;   // units of a row group with eight row tiles
  int64_t span_last;   // units of the last row group
  int64_t span_head;   // units of one kv head: (rg - 1) span_full + span_last
};
__host__ __device__ inline LargeSpans large_spans(const SeqInfo& si, int G) {
  LargeSpans ls;
  const int rows_last = si.n * G - (si.rg - 1) * kLargeRows;
  ls.cost_last = kLargeTileCost[rows_last > 0 ? (rows_last + 31) / 32 : 0];
  const bool any = si.tiles > 0 && si.rg > 0;
  ls.span_full = any ? (int64_t)si.tiles * kLargeTileCost[kLargeRows / 32] : 0;
  ls.span_last = any ? (int64_t)si.tiles * ls.cost_last : 0;
  ls.span_head = any ? (si.rg - 1) * ls.span_full + ls.span_last : 0;
  return ls;
}
// Units of the whole sequence (classes 0 and 1: its tiles per kv head; class 2: in the cost currency).
__host__ __device__ inline int64_t sequence_units(const SeqInfo& si, int cls, int G, int Hkv) {
  if (cls < 2) return (int64_t)si.tiles * Hkv * si.rg;
  return large_spans(si, G).span_head * Hkv;
}
// Tile of a class-2 segment at which a share that begins `off` units into the segment begins (a share boundary
// inside a tile goes down to the tile's beginning).
__host__ __device__ inline int large_tile_at(int64_t off, int cost, int tiles) {
  const int64_t t = off / cost;
  return t > tiles ? tiles : (int)t;
}
// First unit of worker w of W over U units (w = W: U).  Every piece of code that cuts the unit space of class 2
// calls this one function, so that workers and the combine step agree on the pieces.
__host__ __device__ inline int64_t share_begin(int64_t w, int64_t U, int64_t W) { return (w * U) / W; }

// Segments (partial-result slot groups) per class that the host left room for.
struct SegCaps {
  int64_t segs[kClasses];
};

struct PlanView {
  int64_t* header;               // [2c] units U_c, [2c+1] workers W_c, [6+c] first workgroup of class c
  int64_t* cum_units[kClasses];  // [B+1] per class: units before sequence b
  int32_t* cum_segs[kClasses];   // [B+1] per class: segments before sequence b
  int32_t* cum_chunks;    // [B+1] combine row chunks before sequence b
  SeqInfo* info;          // [B]
};

__host__ __device__ inline size_t plan_bytes_for(int batch) {
  const size_t n = (size_t)batch + 2;
  return sizeof(int64_t) * (16 + kClasses * n) + sizeof(SeqInfo) * (size_t)batch +
         sizeof(int32_t) * (kClasses + 1) * n + 64;
}

__host__ __device__ inline PlanView plan_view(void* base, int batch) {
  PlanView v;
  const size_t n = (size_t)batch + 2;
  char* p = (char*)base;
  v.header = (int64_t*)p;
  p += sizeof(int64_t) * 16;
  for (int c = 0; c < kClasses; ++c) {
    v.cum_units[c] = (int64_t*)p;
    p += sizeof(int64_t) * n;
  }
  v.info = (SeqInfo*)p;
  p += sizeof(SeqInfo) * (size_t)batch;
  for (int c = 0; c < kClasses; ++c) {
    v.cum_segs[c] = (int32_t*)p;
    p += sizeof(int32_t) * n;
  }
  v.cum_chunks = (int32_t*)p;
  return v;
}

__host__ __device__ inline int seq_class(int rows) { return rows <= kSmallRows ? 0 : (rows <= kMediumRows ? 1 : 2); }
// With an fp8 cache there is no class 0: trees of up to 64 rows are class 1 (streamed into registers, one or two row
// tiles), larger ones class 2 (tiles staged in LDS as for bf16, after conversion).
template <bool kFp8>
__host__ __device__ inline int plan_class(int rows) {
  return kFp8 ? (rows <= kMediumRows ? 1 : 2) : seq_class(rows);
}

__device__ inline int64_t readlane64(int64_t v, int lane) {
  const uint32_t lo = __builtin_amdgcn_readlane((uint32_t)v, lane);
  const uint32_t hi = __builtin_amdgcn_readlane((uint32_t)((uint64_t)v >> 32), lane);
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// A value every lane agrees on, moved to scalar registers.
__device__ inline int64_t uniform64(int64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
  return (int64_t)(((uint64_t)hi << 32) | lo);
}

// Inclusive add scan over the 64 lanes with data-parallel-primitive moves (no LDS traffic):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of rows 0 and 2 is added to
// rows 1 and 3, then lane 31 to the upper half.  Lanes without a source add zero.
template <int kCtrl, int kRowMask>
__device__ inline int64_t dpp_add(int64_t v) {
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)v, kCtrl, kRowMask, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(uint32_t)((uint64_t)v >> 32), kCtrl, kRowMask, 0xf, false);
  return v + (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// One wavefront: exclusive scan of v and (uniform) the total.
__device__ inline int64_t wave_excl_scan(int64_t v, int lane, int64_t* total) {
  int64_t incl = v;
  incl = dpp_add<0x111, 0xf>(incl);  // row_shr:1
  incl = dpp_add<0x112, 0xf>(incl);  // row_shr:2
  incl = dpp_add<0x114, 0xf>(incl);  // row_shr:4
  incl = dpp_add<0x118, 0xf>(incl);  // row_shr:8
  incl = dpp_add<0x142, 0xa>(incl);  // row_bcast:15 into rows 1 and 3
  incl = dpp_add<0x143, 0xc>(incl);  // row_bcast:31 into rows 2 and 3
  *total = readlane64(incl, kWave - 1);
  return incl - v;
}

// What the plan records of one sequence: lengths and sizes clamped to what the arrays hold.  The
// offsets themselves are checked by offsets_malformed for the whole batch: only a running sum
// guarantees that the sizes add up to at most total_nodes, which is what the host sized the
// partial-result slots and the combine grid for.
// (The row groups are the same with an fp8 cache: one up to 64 rows, else groups of 256.)
template <bool kAllMedium = false>
__device__ inline SeqInfo sequence_info(int len, int base, int next, int total_nodes, int G, int max_blocks) {
  const int cap = max_blocks * kBlock;
  len = len < 0 ? 0 : (len > cap ? cap : len);
  int n = next - base;
  if (base < 0 || n < 0 || base + n > total_nodes) n = 0;
  n = n > SMART_MAX_NODES ? SMART_MAX_NODES : n;
  const int rows = n * G;
  SeqInfo si;
  si.len = len;
  si.n = n;
  si.tiles = (len + kTile - 1) / kTile;
  si.rg = rows == 0 ? 0 : (rows <= kMediumRows ? 1 : (rows + kLargeRows - 1) / kLargeRows);
  return si;
}

// cu_nodes must be a running sum: 0 <= cu[b] <= cu[b + 1] <= total_nodes for every b.  Otherwise the
// sizes of overlapping ranges could add up to more than total_nodes, the bound every buffer of the
// call was sized by; such a batch is planned as if every tree were empty (no output row is written).
__device__ inline bool offsets_malformed(int base, int next, int total_nodes) {
  return base < 0 || next < base || next > total_nodes;
}

// The prefix kernel is ONE launch of max(workgroups, kClasses) workgroups; the classes share
// them in proportion to their cost (kClassTileCost per tile of classes 0 and 1; the units of class 2
// are costs already), so that all of them finish together.  Every class with work gets at least one
// workgroup, the shares are rounded down, and what is left over goes to the classes whose workgroups
// are loaded most, so the classes never need more workgroups than were launched.  Returns the workers
// per class and the first workgroup of each class (entry kClasses: one past the last).
// kOnlySmall: the plan of the fp8-cache kernel, which has no class 0 (plan_class).
template <bool kOnlySmall = false>
__device__ inline void apportion(const int64_t (&all_u)[kClasses], int workgroups, int64_t (&workers)[kClasses],
                                 int64_t (&first_wg)[kClasses + 1]) {
  const int64_t tot_u[kClasses] = {kOnlySmall ? 0 : all_u[0], all_u[1], all_u[2]};
  // (fp8 cache: class 1 is the register stream of half as many bytes per tile; measured 4 .. 8 units per tile
  // against class 2's 11 .. 17, the higher figure where the whole launch is bound by memory)
  const int64_t weight[kClasses] = {kClassTileCost[0], kOnlySmall ? kFp8StreamTileCost : kClassTileCost[1],
                                    kClassTileCost[2]};
  const int64_t launched = workgroups > kClasses ? workgroups : kClasses;
  int64_t cost[kClasses], total = 0;
#pragma unroll
  for (int c = 0; c < kClasses; ++c) {
    cost[c] = tot_u[c] * weight[c];
    total += cost[c];
  }
  int64_t wg[kClasses], used = 0;
  int biggest = 0;
#pragma unroll
  for (int c = 0; c < kClasses; ++c) {
    // (binary64 division: exact enough for a share of a few hundred workgroups, far cheaper than
    // a 64-bit integer division, and every wavefront that plans runs this same code)
    wg[c] = tot_u[c] > 0 ? (int64_t)((double)cost[c] * (double)launched / (double)(total > 0 ? total : 1)) : 0;
    if (tot_u[c] > 0 && wg[c] < 1) wg[c] = 1;
    used += wg[c];
    if (cost[c] > cost[biggest]) biggest = c;
  }
  // What the rounding left over (fewer than kClasses workgroups) goes one by one to the class whose workgroups carry
  // the most cost each: the kernel ends with its slowest class, and a class of four workgroups that is owed 4.5 runs
  // 12 % longer than the rest.  At most kClasses - 1 shares were raised to one, which the biggest class gives back.
  int64_t rest = launched - used;
  for (int k = 0; k < kClasses && rest > 0; ++k) {
    int worst = -1;
#pragma unroll
    for (int c = 0; c < kClasses; ++c)
      if (tot_u[c] > 0 && (worst < 0 || (double)cost[c] * (double)wg[worst] > (double)cost[worst] * (double)wg[c])) worst = c;
    if (worst < 0) break;
    wg[worst] += 1;
    rest -= 1;
  }
#pragma unroll
  for (int c = 0; c < kClasses; ++c)
    if (c == biggest && wg[c] + rest >= 1) wg[c] += rest;
  int64_t first = 0;
#pragma unroll
  for (int c = 0; c < kClasses; ++c) {
    int64_t w = wg[c];  // a worker is a workgroup in every class
    const int64_t cap = tot_u[c] / (kMinTilesPerWorker[c] * (c == 2 ? kLargeTileCost[0] : 1));
    if (w > cap) w = cap;
    if (tot_u[c] > 0 && w < 1) w = 1;
    workers[c] = w;
    first_wg[c] = first;
    first += w;
  }
  first_wg[kClasses] = first;
}

template <bool kOnlySmall>
__global__ __launch_bounds__(kWave) void tva_plan_kernel(
    void* plan_base, int batch, int total_nodes, int G, int Hkv, int max_blocks, int workgroups,
    SegCaps caps, const int32_t* __restrict__ prefix_len, const int32_t* __restrict__ cu_nodes) {
  PlanView pv = plan_view(plan_base, batch);
  const int t = threadIdx.x;
  const int per = (batch + kWave - 1) / kWave;
  const int b0 = min(batch, t * per), b1 = min(batch, b0 + per);
  bool bad = false;
  for (int b = b0; b < b1; ++b) bad = bad || offsets_malformed(cu_nodes[b], cu_nodes[b + 1], total_nodes);
  const bool malformed = __any(bad);
  int64_t units[kClasses] = {0, 0, 0}, segs[kClasses] = {0, 0, 0}, chunks = 0;
  for (int b = b0; b < b1; ++b) {
    SeqInfo si = sequence_info<kOnlySmall>(prefix_len[b], cu_nodes[b], cu_nodes[b + 1], total_nodes, G, max_blocks);
    if (malformed) si.n = si.rg = 0;
    pv.info[b] = si;
    const int rows = si.n * G;
    const int c = plan_class<kOnlySmall>(rows);
    units[c] += sequence_units(si, c, G, Hkv);
    segs[c] += Hkv * si.rg;
    chunks += Hkv * ((rows + kCombineRows - 1) / kCombineRows);
  }
  int64_t tot_u[kClasses], tot_s[kClasses], tot_c, u[kClasses], s[kClasses];
  for (int c = 0; c < kClasses; ++c) {
    u[c] = wave_excl_scan(units[c], t, &tot_u[c]);
    s[c] = wave_excl_scan(segs[c], t, &tot_s[c]);
  }
  int64_t ch = wave_excl_scan(chunks, t, &tot_c);
  // more segments than the host left room for (it sized by a hint that does not hold): nothing runs
  const bool over = tot_s[0] > caps.segs[0] || tot_s[1] > caps.segs[1] || tot_s[2] > caps.segs[2];
  if (over) {
    for (int c = 0; c < kClasses; ++c) tot_u[c] = tot_s[c] = u[c] = s[c] = 0;
    tot_c = ch = 0;
  }
  if (t == 0) {
    int64_t workers[kClasses], first_wg[kClasses + 1];
    apportion<kOnlySmall>(tot_u, workgroups, workers, first_wg);
    for (int c = 0; c < kClasses; ++c) {
      pv.cum_units[c][batch] = tot_u[c];
      pv.cum_segs[c][batch] = (int32_t)tot_s[c];
      pv.header[2 * c] = tot_u[c];
      pv.header[2 * c + 1] = workers[c];
      pv.header[6 + c] = first_wg[c];
    }
    pv.header[6 + kClasses] = first_wg[kClasses];
    pv.cum_chunks[batch] = (int32_t)tot_c;
  }
  for (int b = b0; b < b1; ++b) {
    SeqInfo si = pv.info[b];
    if (over) {
      si.n = si.rg = 0;
      pv.info[b] = si;
    }
    const int rows = si.n * G;
    const int c = plan_class<kOnlySmall>(rows);
    for (int k = 0; k < kClasses; ++k) {
      pv.cum_units[k][b] = u[k];
      pv.cum_segs[k][b] = (int32_t)s[k];
    }
    pv.cum_chunks[b] = (int32_t)ch;
    u[c] += sequence_units(si, c, G, Hkv);
    s[c] += Hkv * si.rg;
    ch += Hkv * ((rows + kCombineRows - 1) / kCombineRows);
  }
}

// The same plan for a batch of at most 64 sequences, computed by a wavefront for itself: lane
// b holds sequence b (lanes past the batch: an empty sequence, so their prefix sums are the
// totals).  One round trip to memory and a few shuffle scans replace a kernel launch.
struct LanePlan {
  SeqInfo si;                   // per lane
  int32_t cu;                   // cu_nodes[lane]
  int64_t cum_units[kClasses];  // per lane: units before this sequence
  int32_t cum_segs[kClasses];
  int32_t cum_chunks;
  int64_t units[kClasses];      // uniform: totals
  int32_t total_segs[kClasses];
  int64_t workers[kClasses];
  int64_t first_wg[kClasses + 1];
  int32_t chunks;
};

template <bool kOnlySmall = false>
__device__ inline void lane_plan(LanePlan& p, const int32_t* prefix_len, const int32_t* cu_nodes, int batch,
                                 int total_nodes, int G, int Hkv, int max_blocks, int workgroups,
                                 const SegCaps& caps, int lane) {
  const int b = min(lane, batch - 1);
  const int32_t len = prefix_len[b], base = cu_nodes[min(lane, batch)], next = cu_nodes[b + 1];
  const bool malformed = __any(lane < batch && offsets_malformed(base, next, total_nodes));
  SeqInfo si = sequence_info<kOnlySmall>(len, base, next, total_nodes, G, max_blocks);
  if (lane >= batch) si.len = si.n = si.tiles = si.rg = 0;
  if (malformed) si.n = si.rg = 0;
  p.cu = base;
  // (a second pass only if the first finds more segments than the host left room for: it sized by a
  // hint that does not hold; then nothing runs)
  for (int pass = 0; pass < 2; ++pass) {
    const int rows = si.n * G;
    const int cls = plan_class<kOnlySmall>(rows);
    const int64_t my_units = sequence_units(si, cls, G, Hkv);
    const int64_t my_segs = Hkv * si.rg;
    int64_t tot_s, tot_c;
#pragma unroll
    for (int c = 0; c < kClasses; ++c) {
      p.cum_units[c] = wave_excl_scan(cls == c ? my_units : 0, lane, &p.units[c]);
      p.cum_segs[c] = (int32_t)wave_excl_scan(cls == c ? my_segs : 0, lane, &tot_s);
      p.total_segs[c] = (int32_t)tot_s;
    }
    p.cum_chunks = (int32_t)wave_excl_scan((int64_t)Hkv * ((rows + kCombineRows - 1) / kCombineRows), lane, &tot_c);
    p.chunks = (int32_t)tot_c;
    if (p.total_segs[0] <= caps.segs[0] && p.total_segs[1] <= caps.segs[1] && p.total_segs[2] <= caps.segs[2]) break;
    si.n = si.rg = 0;
  }
  p.si = si;
  apportion<kOnlySmall>(p.units, workgroups, p.workers, p.first_wg);
}

// ---------------------------------------------------------------------------
// prefix kernels
// ---------------------------------------------------------------------------
struct MainArgs {
  const __bf16* q;
  const __bf16* k_cache;
  const __bf16* v_cache;
  const int32_t* block_table;
  const int32_t* cu_nodes;
  const int32_t* prefix_len;
  void* plan;  // written by the planning kernel; unused for batches of at most 64 sequences
  float* ws[3];  // partial slots per class
  int64_t block_stride, head_stride;
  int32_t batch, total_nodes, Hq, Hkv, G, max_blocks, num_blocks, workgroups;
  SegCaps caps;  // segments per class the partial-result slots have room for
  float scale_log2e;
  // fp8 cache only: k_cache / v_cache then point at bytes (E4M3), scale_log2e already includes k_scale,
  // a partial's row maxima are multiplied by m_scale (= k_scale) and its O by o_scale (= v_scale)
  float m_scale, o_scale;
};

// Wave-uniform data (block table, plan) is read through the constant address
// space so that the loads are scalar and stay off the vector-memory queue the
// K/V stream uses.  Nothing read this way is written by the same kernel.
typedef const __attribute__((address_space(4))) int32_t* const_i32;
typedef const __attribute__((address_space(4))) int64_t* const_i64;
__device__ inline int32_t sload(const int32_t* p) { return *(const_i32)(uintptr_t)p; }
__device__ inline int64_t sload(const int64_t* p) { return *(const_i64)(uintptr_t)p; }
__device__ inline SeqInfo sload(const SeqInfo* p) {
  SeqInfo si;
  const int32_t* q = (const int32_t*)p;
  si.len = sload(q);
  si.n = sload(q + 1);
  si.tiles = sload(q + 2);
  si.rg = sload(q + 3);
  return si;
}

// Row m of a 16-row half of the score tile holds cache slot sigma(m): swapping
// bits 2 and 3 makes the 8 accumulator registers a lane ends up with (rows
// 4h..4h+3 and 8+4h..8+4h+3 of each half) cover 8 consecutive slots, which is
// one V vector of the interleaved layout.
__device__ inline int sigma(int m) { return (m & 3) | ((m & 4) << 1) | ((m & 8) >> 1); }

// Maximum over the two half-wavefronts (lanes j and j + 32) without touching LDS.
__device__ inline float max_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ inline float sum_across_halves(float x) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// Addresses of the two cache pages (one per 16-token block) of a 32-key tile.
struct TilePages {
  int64_t page0, page1;  // element offsets of (block, kv head) pages
};

__device__ inline int64_t clamp_block(int64_t blk, int num_blocks) {
  return blk < 0 ? 0 : (blk >= num_blocks ? num_blocks - 1 : blk);
}

__device__ inline TilePages tile_pages(const MainArgs& a, const int32_t* bt_row, int tile,
                                       int n_blocks, int g) {
  const int i0 = 2 * tile;
  const int i1 = min(2 * tile + 1, n_blocks - 1);  // a missing second block is fully masked later
  TilePages tp;
  tp.page0 = clamp_block(sload(bt_row + i0), a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  tp.page1 = clamp_block(sload(bt_row + i1), a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  return tp;
}

// A load of cache contents that this call reads once (kStream: marked nontemporal) or that another wavefront or a
// later row group reads again (left to the caches).
template <bool kStream, typename T>
__device__ inline T stream_load(const T* p) {
  if (kStream) return __builtin_nontemporal_load(p);
  return *p;
}

// K tile as the A operand of the score product: lane (h, j) holds key row j,
// head dims 16 ks + 8 h .. + 7 for k step ks.
template <bool kStream>
__device__ inline void load_k(bf16x8 (&k)[8], const MainArgs& a, const TilePages& tp, int lane) {
  const int h = lane >> 5, j = lane & 31;
  // rows 0..15 come from the tile's first cache block, rows 16..31 from its second
  // (branch-free select: mask is all ones for the second block)
  const int64_t mask = -(int64_t)(j >> 4);
  const int64_t page = tp.page0 ^ ((tp.page0 ^ tp.page1) & mask);
  const __bf16* kp = a.k_cache + page + (h * 16 + sigma(j & 15)) * 8;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k[ks] = stream_load<kStream>((const bf16x8*)(kp + ks * 256));
}

// V tile as the A operand of the output product: lane (h, j) holds head dim
// 32 jt + j, tokens 8 h .. 8 h + 7 of cache block kk.
template <bool kStream>
__device__ inline void load_v(bf16x8 (&v)[2][4], const MainArgs& a, const TilePages& tp, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const __bf16* vp0 = a.v_cache + tp.page0 + (h * kD + j) * 8;
  const __bf16* vp1 = a.v_cache + tp.page1 + (h * kD + j) * 8;
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    v[0][jt] = stream_load<kStream>((const bf16x8*)(vp0 + jt * 256));
    v[1][jt] = stream_load<kStream>((const bf16x8*)(vp1 + jt * 256));
  }
}

// The same two tiles out of an fp8 cache: the pages have the same element order, one byte per
// element, so a lane's operand vector is 8 bytes; it becomes bf16 (exactly) just before its MFMA.
typedef __attribute__((ext_vector_type(2))) uint32_t fp8x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;

template <bool kStream>
__device__ inline void load_k(fp8x8 (&k)[8], const MainArgs& a, const TilePages& tp, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const int64_t mask = -(int64_t)(j >> 4);
  const int64_t page = tp.page0 ^ ((tp.page0 ^ tp.page1) & mask);
  const uint8_t* kp = (const uint8_t*)a.k_cache + page + (h * 16 + sigma(j & 15)) * 8;
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) k[ks] = stream_load<kStream>((const fp8x8*)(kp + ks * 256));
}

template <bool kStream>
__device__ inline void load_v(fp8x8 (&v)[2][4], const MainArgs& a, const TilePages& tp, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const uint8_t* vp0 = (const uint8_t*)a.v_cache + tp.page0 + (h * kD + j) * 8;
  const uint8_t* vp1 = (const uint8_t*)a.v_cache + tp.page1 + (h * kD + j) * 8;
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    v[0][jt] = stream_load<kStream>((const fp8x8*)(vp0 + jt * 256));
    v[1][jt] = stream_load<kStream>((const fp8x8*)(vp1 + jt * 256));
  }
}

__device__ inline bf16x8 operand(const bf16x8& x) { return x; }
__device__ inline bf16x8 operand(const fp8x8& x) {
  const bf16x2 a = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x[0], 1.0f, false);
  const bf16x2 b = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x[0], 1.0f, true);
  const bf16x2 c = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x[1], 1.0f, false);
  const bf16x2 d = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x[1], 1.0f, true);
  bf16x8 r;
  r[0] = a[0]; r[1] = a[1]; r[2] = b[0]; r[3] = b[1];
  r[4] = c[0]; r[5] = c[1]; r[6] = d[0]; r[7] = d[1];
  return r;
}

__device__ inline void zero_token(bf16x8& v, int e) { v[e] = (__bf16)0.f; }
__device__ inline void zero_token(fp8x8& v, int e) { v[e >> 2] &= ~(0xFFu << (8 * (e & 3))); }  // byte 0x00 = +0

// Masks the ragged end of a prefix: scores of tokens >= n_valid become -inf and
// their V entries zero (unused cache slots may hold anything, NaN included).
template <typename Raw>
__device__ inline void mask_tail(floatx16& s, Raw (&v)[2][4], int n_valid, int h) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * h + (r & 3);  // score-tile row of this register
    const int tok = (i & 16) + sigma(i & 15);      // token of the tile it holds
    if (tok >= n_valid) s[r] = -INFINITY;
  }
#pragma unroll
  for (int kk = 0; kk < 2; ++kk)
#pragma unroll
    for (int e = 0; e < 8; ++e)
      if (kk * 16 + h * 8 + e >= n_valid) {
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) zero_token(v[kk][jt], e);
      }
}

// Online-softmax update of one 32-row tile: scores s (keys x rows, transposed)
// -> bf16 probabilities in the operand layout of the output product.
__device__ inline void softmax_tile(const floatx16& s, float& m, float& l, floatx16 (&o)[4],
                                    bf16x8& pb0, bf16x8& pb1, float c) {
  float mx = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
  mx = max_across_halves(mx);
  const float m_new = fmaxf(m, mx);
  if (__any((m_new - m) * c > kRescaleStep)) {  // the reference follows the maximum in steps: see kRescaleStep
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
    l *= alpha;
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) o[jt] *= alpha;
    m = m_new;
  }
  const float mc = m * c;
  floatx8 p0, p1;
  float sum = 0.f;
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    p0[r] = __builtin_amdgcn_exp2f(fmaf(s[r], c, -mc));
    p1[r] = __builtin_amdgcn_exp2f(fmaf(s[r + 8], c, -mc));
    sum += p0[r] + p1[r];
  }
  l += sum;
  pb0 = __builtin_convertvector(p0, bf16x8);
  pb1 = __builtin_convertvector(p1, bf16x8);
}

// The fold of class 1 stores a partial's 16-byte pieces write-through (device scope) instead of leaving them dirty
// in L2: measured on the workload that is mostly class 1 and bound by memory (64 sequences, prefix 16384), the
// prefix kernel takes 692 us instead of 711, three runs each, alternating.  The same policy measured neutral for
// class 0's fold with a bf16 cache and for class 2's partials, and 3 us slower (50 -> 53 us) for the fold of the fp8
// stream, so only class 1 uses it.  The instruction is
// written as assembly (no builtin carries that cache policy for a 16-byte store); the wait states after it are
// what the compiler would insert itself between a store of more than 8 bytes and the next write of its data
// registers.
__device__ inline void store_through(float* dst, floatx4 x) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1\n\ts_nop 3" ::"v"(dst), "v"(x) : "memory");
}

// Writes one 32-row tile of a partial: O as [d / 4][row][4] so that lanes
// write contiguous 16-byte pieces; then the row maxima and sums.
// (fp8 cache: the scores were taken against the raw key bytes and O against the raw value bytes, so the row maxima
// leave multiplied by m_scale = k_scale and O by o_scale = v_scale; both are 1 for a bf16 cache.)
__device__ inline void store_partial(float* slot, int rows_in_slot, int qt, const floatx16 (&o)[4],
                                     float m, float l, int lane, float m_scale = 1.f, float o_scale = 1.f) {
  const int h = lane >> 5, j = lane & 31;
  const float lsum = sum_across_halves(l);
  // One lane-dependent address, formed here, and constant offsets from it: chunk jt * 8 + 2 * r4 + h of the tile
  // lies (jt * 8 + 2 * r4) * 512 bytes behind chunk h.  (Left to itself the compiler kept sixteen 64-bit offsets
  // alive across the whole piece loop, spilled them, and reloaded one before each store -- and a reload waits for
  // every memory operation in flight, the previous store included: 3.7 .. 4.8 us per partial.)
  // (the pointer keeps its global address space through the barrier: a generic one would turn the stores into flat
  // ones, which also count as LDS traffic and would fall among the counted waits of the next piece)
  typedef __attribute__((address_space(1))) float global_float;
  typedef __attribute__((address_space(1))) floatx4 global_floatx4;
  global_float* first = (global_float*)(slot + ((size_t)(qt * 32 + h) * 32 + j) * 4);
  asm volatile("" : "+v"(first));
#pragma unroll
  for (int jt = 0; jt < 4; ++jt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      floatx4 x;
      x[0] = o[jt][4 * r4 + 0] * o_scale;
      x[1] = o[jt][4 * r4 + 1] * o_scale;
      x[2] = o[jt][4 * r4 + 2] * o_scale;
      x[3] = o[jt][4 * r4 + 3] * o_scale;
      *(global_floatx4*)(first + (jt * 8 + 2 * r4) * 32 * 4) = x;
    }
  if (h == 0) {
    global_float* ml = (global_float*)(slot + rows_in_slot * kD + qt * 32 + j);
    asm volatile("" : "+v"(ml));
    ml[0] = m * m_scale;  // (-inf stays -inf)
    ml[rows_in_slot] = lsum;
  }
}

// Locates the sequence that holds unit u0 in one class's unit space.
__device__ inline int find_sequence(const int64_t* cum_units, int batch, int64_t u0) {
  int lo = 0, hi = batch;
  while (hi - lo > 1) {
    const int mid = (lo + hi) >> 1;
    if (sload(cum_units + mid) <= u0) lo = mid; else hi = mid;
  }
  return lo;
}

// ---- class 0: bandwidth-bound kernel, rows <= 32 -----------------------------------------
//
// K and V each have one register buffer.  The loop body is straight-line:
// scores -> request next K -> softmax -> output product -> request next V, so
// each request is in flight during the other half of the iteration and during
// the co-resident wavefront's work (two wavefronts per SIMD).  The last tile
// of a wavefront's share is taken out of the loop and requests nothing (the
// loop body itself has no conditional request, which keeps the hardware wait
// counters exact); within a share longer than 64 tiles, a 64-tile chunk ends on
// a repeated request for its own last tile.
struct SmallState {
  floatx16 o[4];
  float m, l;
};

// Block ids of tiles [tc, tc + 64) of a sequence live in two registers (lane i
// of reg r holds entry 2 tc + 64 r + i); a tile's two ids come out by readlane.
struct BlockIds {
  int32_t lo, hi;
};

__device__ inline TilePages pages_from_ids(const MainArgs& a, const BlockIds& ids, int rel_tile, int g) {
  const int r = 2 * rel_tile;  // even, so both entries sit in the same register
  const int32_t src = r < kWave ? ids.lo : ids.hi;
  const int64_t blk0 = clamp_block(__builtin_amdgcn_readlane(src, r & (kWave - 1)), a.num_blocks);
  const int64_t blk1 = clamp_block(__builtin_amdgcn_readlane(src, (r + 1) & (kWave - 1)), a.num_blocks);
  TilePages tp;
  tp.page0 = blk0 * a.block_stride + (int64_t)g * a.head_stride;
  tp.page1 = blk1 * a.block_stride + (int64_t)g * a.head_stride;
  return tp;
}

// One tile of a share that is not its last: the requests for the next tile go out as soon as the registers they
// refill are free (K after the score product, V after the output product).
template <bool kStream, typename Raw>
__device__ inline void small_tile(SmallState& S, Raw (&k)[8], Raw (&v)[2][4], const bf16x8 (&q)[8],
                                  int lane, float c, const MainArgs& a, const TilePages& next) {
  floatx16 s = (floatx16)(0.f);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(k[ks]), q[ks], s, 0, 0, 0);
  load_k<kStream>(k, a, next, lane);
  bf16x8 pb0, pb1;
  softmax_tile(s, S.m, S.l, S.o, pb0, pb1, c);
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    S.o[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(v[0][jt]), pb0, S.o[jt], 0, 0, 0);
    S.o[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(v[1][jt]), pb1, S.o[jt], 0, 0, 0);
  }
  load_v<kStream>(v, a, next, lane);
}

// The last tile of a share: nothing follows, so nothing is requested (the streamed lines are not kept in L2, a
// repeated request would go to memory again); it is also the only tile that can be ragged (n_valid < 32).
template <typename Raw>
__device__ inline void small_last_tile(SmallState& S, Raw (&k)[8], Raw (&v)[2][4], const bf16x8 (&q)[8],
                                       int lane, float c, int n_valid) {
  floatx16 s = (floatx16)(0.f);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(k[ks]), q[ks], s, 0, 0, 0);
  if (n_valid < kTile) mask_tail(s, v, n_valid, lane >> 5);
  bf16x8 pb0, pb1;
  softmax_tile(s, S.m, S.l, S.o, pb0, pb1, c);
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) {
    S.o[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(v[0][jt]), pb0, S.o[jt], 0, 0, 0);
    S.o[jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(operand(v[1][jt]), pb1, S.o[jt], 0, 0, 0);
  }
}

// kStream: no other wavefront and no later row group reads these tiles (see stream_load).
template <typename Raw = bf16x8, bool kStream = true>
__device__ inline void small_segment(SmallState& S, const MainArgs& a, int b, int g, int base, int t0,
                                     int t1, const SeqInfo si, int lane, int row0 = 0) {
  const int h = lane >> 5, j = lane & 31;
  const int M = si.n * a.G;
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) S.o[jt] = (floatx16)(0.f);
  S.m = -INFINITY;
  S.l = 0.f;
  if (t0 >= t1) return;  // this wavefront has no tile of the piece
  bf16x8 q[8];  // B operand of the score product: query row j, head dims 16 ks + 8 h ..
  {
    const int rho = row0 + j < M ? row0 + j : M - 1;  // padding rows repeat the last real row; never read back
    const int node = base + rho / a.G, head = g * a.G + rho % a.G;
    const __bf16* qp = a.q + ((int64_t)node * a.Hq + head) * kD + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q[ks] = *(const bf16x8*)(qp + ks * 16);
  }
  const int32_t* bt_row = a.block_table + (int64_t)b * a.max_blocks;
  const int n_blocks = (si.len + kBlock - 1) / kBlock;
  const float c = a.scale_log2e;

  for (int tc = t0; tc < t1; tc += kChunkTiles) {
    const int te = min(t1, tc + kChunkTiles);
    BlockIds ids;
    ids.lo = bt_row[min(2 * tc + lane, n_blocks - 1)];
    ids.hi = bt_row[min(2 * tc + kWave + lane, n_blocks - 1)];
    // Both id registers must have landed before the tile stream starts: inside the loop
    // nothing may wait on them, or the wait would also drain the K/V requests in flight.
    asm volatile("" ::"v"(ids.lo), "v"(ids.hi));
    Raw k[8], v[2][4];
    {
      const TilePages first = pages_from_ids(a, ids, 0, g);
      load_k<kStream>(k, a, first, lane);
      load_v<kStream>(v, a, first, lane);
    }
    // The share's last tile (which the sequence's ragged last tile always is, when the share holds it) is taken
    // out of the loop.  A chunk that is not the share's last ends on a repeated request for its own last tile.
    const bool ends_here = te == t1;
    const int loop_end = ends_here ? te - 1 : te;
    int t = tc;
    for (; t < loop_end; ++t) {
      const TilePages next = pages_from_ids(a, ids, min(t + 1, te - 1) - tc, g);
      small_tile<kStream>(S, k, v, q, lane, c, a, next);
    }
    if (ends_here) small_last_tile(S, k, v, q, lane, c, si.len - t * kTile);
  }
}

// A wavefront's running softmax state in LDS: register by register, lane by lane.
constexpr int kStateFloats = (64 + 2) * kWave;  // 64 accumulator registers + max + sum, per lane

// (four registers of a lane lie together: 16-byte LDS accesses on both sides of the fold)
__device__ inline void state_to_lds(const SmallState& S, float* region, int lane) {
#pragma unroll
  for (int jt = 0; jt < 4; ++jt)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      floatx4 x;
#pragma unroll
      for (int i = 0; i < 4; ++i) x[i] = S.o[jt][4 * r4 + i];
      ((floatx4*)region)[(jt * 4 + r4) * kWave + lane] = x;
    }
  region[64 * kWave + lane] = S.m;
  region[65 * kWave + lane] = S.l;
}
// Accumulator registers 4 quad .. 4 quad + 3 of a lane out of a state in LDS.
__device__ inline floatx4 state_quad(const float* state, int quad, int lane) {
  return ((const floatx4*)state)[quad * kWave + lane];
}


// The eight running states of a piece become ONE partial: every wavefront puts its state in
// LDS, and after one barrier wavefront w merges accumulator registers 8 w .. 8 w + 7 of the
// eight states (always in wavefront order, so the result does not depend on timing) and
// stores that slice of the partial; wavefront 0 also stores the row maxima and sums.
// kScaled (fp8 cache): the partial leaves in true units, row maxima times m_scale, O times o_scale.
// kSlotRows / qt: the slot holds kSlotRows rows and this is its row tile qt.
// kLoadsInFlight: the caller has global loads outstanding that the barriers must not wait for (the next piece's
// first tile); the barriers then only wait for this wavefront's LDS traffic.
template <bool kScaled = false, int kSlotRows = kSmallRows, bool kLoadsInFlight = false>
__device__ inline void fold_and_store(const SmallState& S, float* lds, float* slot, int wv, int lane, float c,
                                      float m_scale = 1.f, float o_scale = 1.f, int qt = 0) {
  const int h = lane >> 5, j = lane & 31;
  state_to_lds(S, lds + wv * kStateFloats, lane);
  if (kLoadsInFlight)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else
    __syncthreads();
  float mk[kWgWaves], lk[kWgWaves];
#pragma unroll
  for (int k = 0; k < kWgWaves; ++k) {
    mk[k] = lds[k * kStateFloats + 64 * kWave + lane];
    lk[k] = lds[k * kStateFloats + 65 * kWave + lane];
  }
  floatx4 part[kWgWaves][2];
#pragma unroll
  for (int k = 0; k < kWgWaves; ++k)
#pragma unroll
    for (int u = 0; u < 2; ++u) part[k][u] = state_quad(lds + k * kStateFloats, 2 * wv + u, lane);
  float m_new = mk[0];
#pragma unroll
  for (int k = 1; k < kWgWaves; ++k) m_new = fmaxf(m_new, mk[k]);
  float l_new = 0.f;
  floatx4 x[2] = {(floatx4)(0.f), (floatx4)(0.f)};
#pragma unroll
  for (int k = 0; k < kWgWaves; ++k) {
    // an empty state has max -inf and contributes nothing
    const float sc = mk[k] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mk[k] - m_new) * c);
    l_new += lk[k] * sc;
    x[0] += part[k][0] * sc;
    x[1] += part[k][1] * sc;
  }
  if (kScaled) {
    x[0] *= o_scale;
    x[1] *= o_scale;
    m_new *= m_scale;  // (-inf stays -inf)
  }
  // accumulator register 16 jt + 4 r4 + i of lane (h, j) is row j, head dims 4 (8 jt + 2 r4 + h) + i
  const int jt = wv >> 1, r4 = 2 * (wv & 1);
  *(floatx4*)(slot + ((size_t)(qt * 32 + jt * 8 + 2 * r4 + h) * 32 + j) * 4) = x[0];
  *(floatx4*)(slot + ((size_t)(qt * 32 + jt * 8 + 2 * (r4 + 1) + h) * 32 + j) * 4) = x[1];
  if (wv == 0) {
    const float lsum = sum_across_halves(l_new);
    if (h == 0) {
      slot[kSlotRows * kD + qt * 32 + j] = m_new;
      slot[kSlotRows * kD + kSlotRows + qt * 32 + j] = lsum;
    }
  }
  // the next piece reuses the LDS regions
  if (kLoadsInFlight)
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
  else
    __syncthreads();
}

// The plan entries of 64 consecutive sequences, one per lane, fetched with one
// round trip; a worker's range rarely leaves the window it starts in.
struct PlanWindow {
  int first;          // sequence held by lane 0
  int64_t cum_units;  // lane i: units before sequence first + i (entry `batch` included)
  int32_t cum_segs;
  int32_t cu_nodes;
  int32_t len, n, tiles, rg;
  int64_t total_units;  // entry 64 of a window that holds a whole batch of 64 (uniform)
};

// Units before the sequence at window index i (0 .. 64).
__device__ inline int64_t window_cum_units(const PlanWindow& w, int i) {
  return i < kWave ? readlane64(w.cum_units, i) : w.total_units;
}

// A workgroup's copy of the plan when its first wavefront derived it (batches of at most 64).
struct PlanShare {
  int64_t cum_units[kClasses][kWave];
  int32_t cum_segs[kClasses][kWave];
  int32_t cu[kWave];
  SeqInfo info[kWave];
  int64_t units[kClasses], workers[kClasses], first_wg[kClasses + 1];
};

__device__ inline void load_window(PlanWindow& w, const PlanView& pv, const int32_t* cu_nodes,
                                   int cls, int batch, int first, int lane) {
  w.first = first;
  const int e = min(first + lane, batch);      // entries 0 .. batch exist
  const int b = min(first + lane, batch - 1);  // per-sequence info exists for 0 .. batch - 1
  w.cum_units = pv.cum_units[cls][e];
  w.cum_segs = pv.cum_segs[cls][e];
  w.cu_nodes = cu_nodes[e];
  const SeqInfo si = pv.info[b];
  w.len = si.len;
  w.n = si.n;
  w.tiles = si.tiles;
  w.rg = si.rg;
  w.total_units = 0;  // never read: such a window is reloaded before its last lane is passed
}

__device__ inline SeqInfo window_info(const PlanWindow& w, int b) {
  const int i = b - w.first;
  SeqInfo si;
  si.len = __builtin_amdgcn_readlane(w.len, i);
  si.n = __builtin_amdgcn_readlane(w.n, i);
  si.tiles = __builtin_amdgcn_readlane(w.tiles, i);
  si.rg = __builtin_amdgcn_readlane(w.rg, i);
  return si;
}

// What a worker needs of the plan: its class's unit and worker counts, and the window (held in
// registers for the whole batch when the wavefront planned for itself, else loaded from the
// plan in memory as the worker moves along).
struct ClassPlan {
  int64_t U, W;
  bool resident;
  PlanWindow win;
};

// Sequence that holds unit u0 of class `cls`, with its plan window loaded.
__device__ inline int locate(ClassPlan& cp, const PlanView& pv, const int32_t* cu_nodes, int cls,
                             int batch, int64_t u0, int lane) {
  if (batch <= kWave) {
    if (!cp.resident) load_window(cp.win, pv, cu_nodes, cls, batch, 0, lane);
    // cum_units is non-decreasing: the lanes with cum <= u0 are a prefix, its last lane is b
    const uint64_t below = __ballot(lane < batch && cp.win.cum_units <= u0);
    return __popcll(below) - 1;
  }
  const int b = find_sequence(pv.cum_units[cls], batch, u0);
  load_window(cp.win, pv, cu_nodes, cls, batch, b, lane);
  return b;
}

// Moves the window along when sequence b is its last lane (a resident window never moves).
__device__ inline void follow(ClassPlan& cp, const PlanView& pv, const int32_t* cu_nodes, int cls, int batch,
                              int b, int lane) {
  if (!cp.resident && b - cp.win.first >= kWave - 1) load_window(cp.win, pv, cu_nodes, cls, batch, b, lane);
}

// One workgroup of eight wavefronts per worker (two per SIMD).  Worker w owns
// units [w U / W, (w+1) U / W) of class 0; every piece of that range (its
// intersection with one (sequence, kv head) segment) is cut into eight
// contiguous sub-ranges, one per wavefront, and the eight running states are
// folded together through LDS after one barrier (fold_and_store), so that a
// piece leaves ONE partial in memory however many wavefronts streamed it.
constexpr int kSmallWaves = kWgWaves;

// A piece: the part of a worker's unit range that lies in one (sequence, kv head) segment.
struct SmallPiece {
  int b, g, base, t0, nt;
  int64_t seg;
  SeqInfo si;
  bool valid;
};

// The piece that starts at unit u0 of the worker's range [.., u1) (sequences without units of this class are
// skipped; b moves along).
__device__ inline SmallPiece small_piece(ClassPlan& cp, const PlanView& pv, const MainArgs& a, int64_t u0, int64_t u1,
                                         int& b, int lane) {
  SmallPiece p;
  p.valid = false;
  PlanWindow& win = cp.win;
  while (u0 < u1 && b < a.batch) {
    follow(cp, pv, a.cu_nodes, 0, a.batch, b, lane);
    const int64_t seq_begin = window_cum_units(win, b - win.first);
    const int64_t seq_end = window_cum_units(win, b + 1 - win.first);
    if (u0 >= seq_end) { ++b; continue; }
    p.si = window_info(win, b);
    // (the divisions run on the vector unit; everything is wavefront-uniform and goes back to scalar registers)
    const int64_t local = u0 - seq_begin;
    p.b = __builtin_amdgcn_readfirstlane(b);
    p.g = __builtin_amdgcn_readfirstlane((int)(local / p.si.tiles));
    p.t0 = __builtin_amdgcn_readfirstlane((int)(local % p.si.tiles));
    const int64_t left = u1 - u0;
    p.nt = __builtin_amdgcn_readfirstlane((int)(left < (int64_t)(p.si.tiles - p.t0) ? left : (int64_t)(p.si.tiles - p.t0)));
    p.seg = uniform64((int64_t)__builtin_amdgcn_readlane(win.cum_segs, b - win.first) + p.g);
    p.base = __builtin_amdgcn_readlane(win.cu_nodes, b - win.first);
    p.valid = true;
    break;
  }
  return p;
}

// Pulls what a wavefront reads first of its share of piece p into the L2 cache: the share's first K/V tile (128
// lines of 128 bytes: lanes 0..31 the first cache block, 32..63 the second), the block ids of its first 64 tiles and
// the query rows.  One dword per lane and line; the values are not used, only kept until the caller has folded the
// current piece, so the requests are in flight during the fold and the share then starts on L2 hits.
__device__ inline void small_touch(uint32_t (&touched)[4], const MainArgs& a, const SmallPiece& p, int s0, int32_t blk0,
                                   int32_t blk1, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const int64_t page = clamp_block(h ? blk1 : blk0, a.num_blocks) * a.block_stride + (int64_t)p.g * a.head_stride;
  touched[0] = *(const uint32_t*)(a.k_cache + page + j * 64);
  touched[1] = *(const uint32_t*)(a.v_cache + page + j * 64);
  const int32_t* bt_row = a.block_table + (int64_t)p.b * a.max_blocks;
  const int n_blocks = (p.si.len + kBlock - 1) / kBlock;
  touched[2] = (uint32_t)bt_row[min(2 * s0 + 2 * lane, n_blocks - 1)];
  const int M = p.si.n * a.G;
  const int rho = j < M ? j : M - 1;
  const int node = p.base + rho / a.G, head = p.g * a.G + rho % a.G;
  touched[3] = *(const uint32_t*)(a.q + ((int64_t)node * a.Hq + head) * kD + h * 64);
}

__device__ inline void small_worker(const MainArgs& a, int64_t w, ClassPlan& cp, float* merge_lds /* 132 KB: eight states */) {
  const PlanView pv = plan_view(a.plan, a.batch);
  const int64_t U = cp.U, W = cp.W;
  if (w >= W || U <= 0) return;
  int64_t u0 = (w * U) / W;
  const int64_t u1 = ((w + 1) * U) / W;
  if (u0 >= u1) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int b = locate(cp, pv, a.cu_nodes, 0, a.batch, u0, lane);
  SmallPiece cur = small_piece(cp, pv, a, u0, u1, b, lane);
  while (cur.valid) {
    // The piece after this one is located first: what this wavefront will read first of it is requested before
    // the fold of this piece, so that the stream does not start from memory latency at every piece boundary.
    const SmallPiece nxt = small_piece(cp, pv, a, u0 + cur.nt, u1, b, lane);
    // this wavefront's share of the piece, and of the next
    const int s0 = cur.t0 + (int)(((int64_t)cur.nt * wv) / kSmallWaves);
    const int s1 = cur.t0 + (int)(((int64_t)cur.nt * (wv + 1)) / kSmallWaves);
    int n0 = 0, n1 = 0;
    if (nxt.valid) {
      n0 = nxt.t0 + (int)(((int64_t)nxt.nt * wv) / kSmallWaves);
      n1 = nxt.t0 + (int)(((int64_t)nxt.nt * (wv + 1)) / kSmallWaves);
    }
    const bool pre = n0 < n1;
    // block ids of the next share's first tile: scalar loads, issued a whole share ahead
    int32_t nb0 = 0, nb1 = 0;
    if (pre) {
      const int32_t* row = a.block_table + (int64_t)nxt.b * a.max_blocks;
      const int nblk = (nxt.si.len + kBlock - 1) / kBlock;
      nb0 = sload(row + min(2 * n0, nblk - 1));
      nb1 = sload(row + min(2 * n0 + 1, nblk - 1));
    }
    SmallState S;
    small_segment(S, a, cur.b, cur.g, cur.base, s0, s1, cur.si, lane);
    uint32_t touched[4] = {0u, 0u, 0u, 0u};
    if (pre) small_touch(touched, a, nxt, n0, nb0, nb1, lane);
    fold_and_store<false, kSmallRows, true>(S, merge_lds, a.ws[0] + (size_t)(w + cur.seg) * kSmallSlot, wv, lane,
                                            a.scale_log2e);
    asm volatile("" ::"v"(touched[0]), "v"(touched[1]), "v"(touched[2]), "v"(touched[3]));
    u0 += cur.nt;
    cur = nxt;
  }
}

// ---- fp8 cache: every sequence in row groups of up to 64 rows, streamed into registers ---------
//
// The same register-direct stream as class 0.  A row group with more than 32 rows has two row
// tiles, one per half of the workgroup.

// A row group of two row tiles: wavefronts 0..3 carry row tile 0, wavefronts 4..7 row tile 1, each
// half cuts the piece's tiles four ways and both halves stream the SAME tiles (the second request
// for a tile is served by the caches, HBM sees it once).  Their states meet in LDS like the eight
// of a one-tile piece; wavefront w then merges accumulator registers 16 (w % 4) .. + 15 of the four
// states of row tile w / 4 (always in wavefront order) and stores that slice of the 64-row slot.
__device__ inline void fold_halves_and_store(const SmallState& S, float* lds, float* slot, int wv, int lane, float c,
                                             float m_scale, float o_scale) {
  const int h = lane >> 5, j = lane & 31;
  state_to_lds(S, lds + wv * kStateFloats, lane);
  __syncthreads();
  const int rt = wv >> 2, part = wv & 3;
  float mk[4], lk[4];
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    mk[k] = lds[(4 * rt + k) * kStateFloats + 64 * kWave + lane];
    lk[k] = lds[(4 * rt + k) * kStateFloats + 65 * kWave + lane];
  }
  float m_new = fmaxf(fmaxf(mk[0], mk[1]), fmaxf(mk[2], mk[3]));
  float l_new = 0.f;
  floatx4 x[4] = {(floatx4)(0.f), (floatx4)(0.f), (floatx4)(0.f), (floatx4)(0.f)};
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    // an empty state has max -inf and contributes nothing
    const float sc = mk[k] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mk[k] - m_new) * c);
    l_new += lk[k] * sc;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      x[u] += state_quad(lds + (4 * rt + k) * kStateFloats, 4 * part + u, lane) * sc;
    }
  }
  // accumulator register 16 jt + 4 r4 + i of lane (h, j) is row j, head dims 4 (8 jt + 2 r4 + h) + i; here jt = part, r4 = u
#pragma unroll
  for (int u = 0; u < 4; ++u)
    *(floatx4*)(slot + ((size_t)(rt * 32 + part * 8 + 2 * u + h) * 32 + j) * 4) = x[u] * o_scale;
  if (part == 0) {
    const float lsum = sum_across_halves(l_new);
    if (h == 0) {
      slot[kMediumRows * kD + rt * 32 + j] = m_new * m_scale;  // (-inf stays -inf)
      slot[kMediumRows * kD + kMediumRows + rt * 32 + j] = lsum;
    }
  }
  __syncthreads();  // the next piece reuses the LDS regions
}

__device__ inline void fp8_worker(const MainArgs& a, int64_t w, ClassPlan& cp, float* merge_lds /* 132 KB */) {
  const PlanView pv = plan_view(a.plan, a.batch);
  const int64_t U = cp.U, W = cp.W;
  PlanWindow& win = cp.win;
  if (w >= W || U <= 0) return;
  int64_t u0 = (w * U) / W;
  const int64_t u1 = ((w + 1) * U) / W;
  if (u0 >= u1) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int b = locate(cp, pv, a.cu_nodes, 1, a.batch, u0, lane);
  while (u0 < u1 && b < a.batch) {
    follow(cp, pv, a.cu_nodes, 1, a.batch, b, lane);
    const int64_t seq_begin = window_cum_units(win, b - win.first);
    const int64_t seq_end = window_cum_units(win, b + 1 - win.first);
    if (u0 >= seq_end) { ++b; continue; }
    const SeqInfo si = window_info(win, b);
    const int64_t local = u0 - seq_begin;
    const int seg_local = (int)(local / si.tiles);  // kv head x row group of 64 rows
    const int g = seg_local / si.rg;
    const int row0 = (seg_local % si.rg) * kMediumRows;
    const int t0 = (int)(local % si.tiles);
    const int64_t left = u1 - u0;
    const int nt = (int)(left < (int64_t)(si.tiles - t0) ? left : (int64_t)(si.tiles - t0));
    const int64_t seg = (int64_t)__builtin_amdgcn_readlane(win.cum_segs, b - win.first) + seg_local;
    const int base = __builtin_amdgcn_readlane(win.cu_nodes, b - win.first);
    float* slot = a.ws[1] + (size_t)(w + seg) * kMediumSlot;
    SmallState S;
    if (si.n * a.G - row0 <= kSmallRows) {
      const int s0 = t0 + (int)(((int64_t)nt * wv) / kWgWaves);
      const int s1 = t0 + (int)(((int64_t)nt * (wv + 1)) / kWgWaves);
      // a tree with one tile of rows reads every K/V tile once; otherwise the other half of the workgroup or the
      // other row groups read the same tiles again, out of the caches
      if (si.rg == 1)
        small_segment<fp8x8, true>(S, a, b, g, base, s0, s1, si, lane, row0);
      else
        small_segment<fp8x8, false>(S, a, b, g, base, s0, s1, si, lane, row0);
      fold_and_store<true, kMediumRows>(S, merge_lds, slot, wv, lane, a.scale_log2e, a.m_scale, a.o_scale, 0);
    } else {
      const int rt = wv >> 2, sub = wv & 3;
      const int s0 = t0 + (int)(((int64_t)nt * sub) / 4);
      const int s1 = t0 + (int)(((int64_t)nt * (sub + 1)) / 4);
      small_segment<fp8x8, false>(S, a, b, g, base, s0, s1, si, lane, row0 + rt * kSmallRows);
      fold_halves_and_store(S, merge_lds, slot, wv, lane, a.scale_log2e, a.m_scale, a.o_scale);
    }
    u0 += nt;
  }
}

// ---- classes 1 and 2: K/V tiles staged in LDS, shared by the eight wavefronts of a workgroup --
//
// A workgroup of eight wavefronts (two per SIMD) is the worker.  A tile (16 KB: 8 K + 8 V
// operand vectors per lane) is fetched from HBM once per workgroup, each wavefront requesting
// an eighth of it, straight into LDS in operand order -- the vector a lane will feed to the
// MFMA sits at [instruction][lane], so reads are 16 bytes per lane at consecutive addresses,
// free of bank conflicts.
//   class 2 (more than 64 rows): row groups of up to 256 rows, wavefront w carries rows
//     32 w .. 32 w + 31; one tile per iteration and barrier; the score product of the next
//     tile is woven into the softmax of the current one (staged_segment).
//   class 1 (33 .. 64 rows): row tile = w / 2 (tiles 0 and 1 have rows), key group = w % 2;
//     two tiles per iteration, one per key group; the two states of a row tile are folded
//     through LDS at the end of the segment (grouped_segment).
// K/V tiles travel HBM -> LDS without passing through registers (global_load_lds, 16 bytes a
// lane).  A stage holds one 32-key tile in operand order: eight K vectors (k steps) then
// eight V vectors (cache block kk, d tile jt at 4 kk + jt), 64 lanes x 16 bytes each;
// wavefront w fetches vectors 2 w and 2 w + 1 of every tile.  kStages tiles are in flight.
constexpr int kStages = 8;
constexpr int kStageVecs = 16 * kWave;

typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(1))) const void global_void;

__device__ inline uint32_t lds_address(const void* p) { return (uint32_t)(uintptr_t)(lds_void*)p; }

// What a lane fetches of every tile: fixed offset inside a page, and which of the tile's two
// pages (mask all ones: the second).
struct FetchLane {
  const __bf16* base;
  int64_t second_page;
};

__device__ inline FetchLane fetch_lane(const MainArgs& a, int wv, int lane) {
  const int h = lane >> 5, j = lane & 31;
  FetchLane f;
  if (wv < 4) {  // K vectors of k steps 2 wv, 2 wv + 1: key row j, head dims 16 ks + 8 h ..
    f.base = a.k_cache + (h * 16 + sigma(j & 15)) * 8 + wv * 2 * 256;
    f.second_page = -(int64_t)(j >> 4);
  } else {  // V vectors of cache block (wv - 4) / 2, d tiles 2 ((wv - 4) % 2) + {0, 1}
    f.base = a.v_cache + (h * kD + j) * 8 + 2 * ((wv - 4) & 1) * 256;
    f.second_page = -(int64_t)((wv - 4) >> 1);
  }
  return f;
}

// `again`: the tile is requested more than once -- a request past the end of a segment repeats the segment's last
// tile so that every iteration issues the same number of requests (it is never consumed), and a tree with several row
// groups streams the prefix once per group.  Such requests are left cacheable, so that the repeats can hit in L2 or
// the last-level cache instead of going to memory like the read-once stream does.
__device__ inline void request_tile(const MainArgs& a, const FetchLane& f, int32_t blk0, int32_t blk1, int g,
                                    bf16x8* stage, int wv, bool again) {
  const int64_t page0 = clamp_block(blk0, a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  const int64_t page1 = clamp_block(blk1, a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  const __bf16* src = f.base + (page0 ^ ((page0 ^ page1) & f.second_page));
  bf16x8* dst = stage + 2 * wv * kWave;
  if (again) {
    __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)dst, 16, 0, 0);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 256), (lds_void*)(dst + kWave), 16, 0, 0);
  } else {
    __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)dst, 16, 0, kStreamPolicy);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 256), (lds_void*)(dst + kWave), 16, 0, kStreamPolicy);
  }
}

// The same tile out of an fp8 cache.  The pages have the same element order with one byte per element, so the two
// operand vectors a lane is responsible for are 8 bytes each, 256 bytes apart.  They travel HBM -> LDS as four
// dwords per lane (the LDS-direct load takes 4 or 16 bytes a lane) into this wavefront's 1 KB of a raw slot:
// plane p of 64 dwords holds dword p of every lane (vector 0 low, vector 0 high, vector 1 low, vector 1 high).
// convert_tile_fp8 then turns them into the two bf16 operand vectors of the stage, exactly (E4M3 -> bf16).
__device__ inline FetchLane fetch_lane_fp8(const MainArgs& a, int wv, int lane) {
  const int h = lane >> 5, j = lane & 31;
  const uint8_t* kb = (const uint8_t*)a.k_cache;
  const uint8_t* vb = (const uint8_t*)a.v_cache;
  FetchLane f;
  if (wv < 4) {
    f.base = (const __bf16*)(kb + (h * 16 + sigma(j & 15)) * 8 + wv * 2 * 256);
    f.second_page = -(int64_t)(j >> 4);
  } else {
    f.base = (const __bf16*)(vb + (h * kD + j) * 8 + 2 * ((wv - 4) & 1) * 256);
    f.second_page = -(int64_t)((wv - 4) >> 1);
  }
  return f;
}

__device__ inline void request_tile_fp8(const MainArgs& a, const FetchLane& f, int32_t blk0, int32_t blk1, int g,
                                        uint32_t* raw /* this wavefront's 4 x 64 dwords of the slot */, bool again) {
  const int64_t page0 = clamp_block(blk0, a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  const int64_t page1 = clamp_block(blk1, a.num_blocks) * a.block_stride + (int64_t)g * a.head_stride;
  const uint8_t* src = (const uint8_t*)f.base + (page0 ^ ((page0 ^ page1) & f.second_page));
  if (again) {
    __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)raw, 4, 0, 0);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 4), (lds_void*)(raw + kWave), 4, 0, 0);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 256), (lds_void*)(raw + 2 * kWave), 4, 0, 0);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 260), (lds_void*)(raw + 3 * kWave), 4, 0, 0);
  } else {
    __builtin_amdgcn_global_load_lds((global_void*)src, (lds_void*)raw, 4, 0, kStreamPolicy);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 4), (lds_void*)(raw + kWave), 4, 0, kStreamPolicy);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 256), (lds_void*)(raw + 2 * kWave), 4, 0, kStreamPolicy);
    __builtin_amdgcn_global_load_lds((global_void*)(src + 260), (lds_void*)(raw + 3 * kWave), 4, 0, kStreamPolicy);
  }
}

// raw_addr: LDS byte address of this lane's dword in plane 0 of the raw slot; dst_addr: that of its first operand
// vector in the stage (the second is 64 vectors further).  Written as assembly like the operand reads: an LDS access
// the compiler can see makes it wait for every LDS-direct load in flight.  Ends with the writes done.
__device__ inline void convert_tile_fp8(uint32_t raw_addr, uint32_t dst_addr) {
  uint32_t d0, d1, d2, d3;
  asm volatile(
      "ds_read_b32 %0, %4\n\t"
      "ds_read_b32 %1, %4 offset:256\n\t"
      "ds_read_b32 %2, %4 offset:512\n\t"
      "ds_read_b32 %3, %4 offset:768\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(d0), "=&v"(d1), "=&v"(d2), "=&v"(d3)
      : "v"(raw_addr)
      : "memory");
  fp8x8 r0, r1;
  r0[0] = d0, r0[1] = d1, r1[0] = d2, r1[1] = d3;
  const bf16x8 b0 = operand(r0), b1 = operand(r1);
  asm volatile(
      "ds_write_b128 %0, %1\n\t"
      "ds_write_b128 %0, %2 offset:1024\n\t"
      "s_waitcnt lgkmcnt(0)"
      :
      : "v"(dst_addr), "v"(b0), "v"(b1)
      : "memory");
}

// LDS reads of the staged tiles are written as assembly: the compiler would otherwise wait
// for every outstanding global_load_lds before each read it can see.  The counter waits
// below carry the registers they release as operands, so that no use can move above them.
#define SMART_LDS_READ(dst, addr, OFFSET) \
  asm volatile("ds_read_b128 %0, %1 offset:" #OFFSET : "=v"(dst) : "v"(addr) : "memory")
#define SMART_LDS_WAIT(reg, N) asm volatile("s_waitcnt lgkmcnt(" #N ")" : "+v"(reg) : : "memory")

__device__ inline void lds_read_half(bf16x8 (&r)[8], uint32_t addr, int half) {
  if (half == 0) {
    SMART_LDS_READ(r[0], addr, 0);
    SMART_LDS_READ(r[1], addr, 1024);
    SMART_LDS_READ(r[2], addr, 2048);
    SMART_LDS_READ(r[3], addr, 3072);
  } else {
    SMART_LDS_READ(r[4], addr, 4096);
    SMART_LDS_READ(r[5], addr, 5120);
    SMART_LDS_READ(r[6], addr, 6144);
    SMART_LDS_READ(r[7], addr, 7168);
  }
}

// The V fetchers clear the entries of tokens >= n_valid in their two vectors of a landed
// stage (ragged end of a prefix; unowned slots may hold NaN).
__device__ inline void zero_invalid_v_lds(bf16x8* stage, int wv, int lane, int n_valid) {
  if (wv < 4) return;
  const int h = lane >> 5, kk = (wv - 4) >> 1;
  const uint32_t addr = lds_address(stage + 2 * wv * kWave + lane);
  bf16x8 v0, v1;
  SMART_LDS_READ(v0, addr, 0);
  SMART_LDS_READ(v1, addr, 1024);
  SMART_LDS_WAIT(v0, 0);
  SMART_LDS_WAIT(v1, 0);
#pragma unroll
  for (int x = 0; x < 8; ++x)
    if (kk * 16 + h * 8 + x >= n_valid) {
      v0[x] = (__bf16)0.f;
      v1[x] = (__bf16)0.f;
    }
  asm volatile("ds_write_b128 %0, %1\n\tds_write_b128 %0, %2 offset:1024\n\ts_waitcnt lgkmcnt(0)"
               :
               : "v"(addr), "v"(v0), "v"(v1)
               : "memory");
}

__device__ inline void mask_scores(floatx16& s, int n_valid, int h) {
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    const int i = 8 * (r >> 2) + 4 * h + (r & 3);
    const int tok = (i & 16) + sigma(i & 15);
    if (tok >= n_valid) s[r] = -INFINITY;
  }
}

// Scores of one staged tile (used for the first tile of a segment only).
__device__ inline void score_tile(floatx16& s, uint32_t k_addr, const bf16x8 (&q)[8]) {
  bf16x8 kop[8];
  lds_read_half(kop, k_addr, 0);
  lds_read_half(kop, k_addr, 1);
  SMART_LDS_WAIT(kop[0], 0);
  s = (floatx16)(0.f);
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    if (ks > 0) SMART_LDS_WAIT(kop[ks], 0);
    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[ks], q[ks], s, 0, 0, 0);
  }
}

// One iteration of a wavefront with rows: softmax and output product of tile t (scores
// s_in, V at v_addr) with the score product of tile t + 1 (K at k_addr, result s_out) woven
// in, so that the matrix cores run in the shadow of the exponentials:
//   8 x { score MFMA k step i | exp of first-half probability i }
//   4 x { output MFMA (first cache block, d tile jt) | exp of second-half probabilities 2 jt, 2 jt + 1 }
//   4 x   output MFMA (second cache block)
// The scheduling barriers keep that order.  `between` runs after the first LDS reads are
// issued (the caller's fetch requests go there, in the shadow of the LDS latency).  The
// counts of the LDS waits follow the order in which the 16 reads are issued: K 0..7 and
// V 0..3 up front, V 4..7 after the fourth score step.
template <typename Between>
__device__ inline void woven_tile(const floatx16& s, floatx16& s_next, floatx16 (&o)[4], float& m, float& l,
                                  const bf16x8 (&q)[8], uint32_t k_addr, uint32_t v_addr, float c,
                                  Between between) {
  bf16x8 kop[8], vop[8];
  lds_read_half(kop, k_addr, 0);
  lds_read_half(kop, k_addr, 1);
  lds_read_half(vop, v_addr, 0);
  between();
  float mx = s[0];
#pragma unroll
  for (int r = 1; r < 16; ++r) mx = fmaxf(mx, s[r]);
  mx = max_across_halves(mx);
  const float m_new = fmaxf(m, mx);
  if (__any((m_new - m) * c > kRescaleStep)) {  // the reference follows the maximum in steps: see kRescaleStep
    const float alpha = __builtin_amdgcn_exp2f((m - m_new) * c);
    l *= alpha;
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) o[jt] *= alpha;
    m = m_new;
  }
  const float mc = m * c;
  s_next = (floatx16)(0.f);
  floatx8 p0, p1;
  float sum = 0.f;
  __builtin_amdgcn_sched_barrier(0);
#define SMART_SCORE_STEP(I, N)                                                        \
  SMART_LDS_WAIT(kop[I], N);                                                          \
  s_next = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[I], q[I], s_next, 0, 0, 0);    \
  p0[I] = __builtin_amdgcn_exp2f(fmaf(s[I], c, -mc));                                 \
  sum += p0[I];                                                                       \
  __builtin_amdgcn_sched_barrier(0);
  SMART_SCORE_STEP(0, 11)
  SMART_SCORE_STEP(1, 10)
  SMART_SCORE_STEP(2, 9)
  SMART_SCORE_STEP(3, 8)
  lds_read_half(vop, v_addr, 1);  // outstanding: K 4..7, V 0..7
  SMART_SCORE_STEP(4, 11)
  SMART_SCORE_STEP(5, 10)
  SMART_SCORE_STEP(6, 9)
  SMART_SCORE_STEP(7, 8)
#undef SMART_SCORE_STEP
  const bf16x8 pb0 = __builtin_convertvector(p0, bf16x8);
  __builtin_amdgcn_sched_barrier(0);
#define SMART_OUTPUT_STEP(JT, N)                                                      \
  SMART_LDS_WAIT(vop[JT], N);                                                         \
  o[JT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[JT], pb0, o[JT], 0, 0, 0);      \
  p1[2 * JT] = __builtin_amdgcn_exp2f(fmaf(s[8 + 2 * JT], c, -mc));                   \
  p1[2 * JT + 1] = __builtin_amdgcn_exp2f(fmaf(s[9 + 2 * JT], c, -mc));               \
  sum += p1[2 * JT] + p1[2 * JT + 1];                                                 \
  __builtin_amdgcn_sched_barrier(0);
  SMART_OUTPUT_STEP(0, 7)
  SMART_OUTPUT_STEP(1, 6)
  SMART_OUTPUT_STEP(2, 5)
  SMART_OUTPUT_STEP(3, 4)
#undef SMART_OUTPUT_STEP
  l += sum;
  const bf16x8 pb1 = __builtin_convertvector(p1, bf16x8);
  SMART_LDS_WAIT(vop[4], 3);
  o[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[4], pb1, o[0], 0, 0, 0);
  SMART_LDS_WAIT(vop[5], 2);
  o[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[5], pb1, o[1], 0, 0, 0);
  SMART_LDS_WAIT(vop[6], 1);
  o[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[6], pb1, o[2], 0, 0, 0);
  SMART_LDS_WAIT(vop[7], 0);
  o[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[7], pb1, o[3], 0, 0, 0);
}

// All eight wavefronts of the workgroup run this together (it contains barriers);
// kRows = false marks a wavefront without rows in this row group: it only helps to fetch.
// kFp8: the cache holds E4M3 bytes.  LDS then holds four bf16 stages (a tile is used during two iterations) and,
// behind them, kStages raw slots of 8 KB; a wavefront converts its own share of tile t + 1 as soon as it has
// landed (nobody else touches those bytes), before the barrier that publishes the stage.
template <bool kRows, bool kFp8 = false>
__device__ inline void staged_segment(const MainArgs& a, int b, int g, int base, int row0, int t0, int t1,
                                      const SeqInfo si, float* slot, int wv, int lane, bf16x8* lds) {
  constexpr int kRing = kFp8 ? 4 : kStages;  // bf16 stages
  constexpr int kLoads = kFp8 ? 4 : 2;       // vector-memory loads per tile and wavefront
  const int h = lane >> 5, j = lane & 31;
  const int M = si.n * a.G;
  floatx16 o[4];
  bf16x8 q[8];
  float m = -INFINITY, l = 0.f;
  if (kRows) {
    int rho = row0 + j;
    rho = rho < M ? rho : M - 1;  // padding rows repeat the last real row; never read back
    const int node = base + rho / a.G, head = g * a.G + rho % a.G;
    const __bf16* qp = a.q + ((int64_t)node * a.Hq + head) * kD + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q[ks] = *(const bf16x8*)(qp + ks * 16);
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) o[jt] = (floatx16)(0.f);
    // (not waited for here: the tile requests below are younger loads, so the wait for the first tile covers these)
  }
  const int32_t* bt_row = a.block_table + (int64_t)b * a.max_blocks;
  const int n_blocks = (si.len + kBlock - 1) / kBlock;
  const float c = a.scale_log2e;
  const FetchLane f = kFp8 ? fetch_lane_fp8(a, wv, lane) : fetch_lane(a, wv, lane);
  const uint32_t rd = lds_address(lds + lane);  // this lane's slice of vector 0 of stage 0
  const int last = t1 - 1;
  auto stage_of = [&](int t) { return lds + (t & (kRing - 1)) * kStageVecs; };
  // fp8: this wavefront's 4 x 64 dwords of tile t's raw slot, and the conversion of its share of tile t
  uint32_t* const raw_base = (uint32_t*)(lds + kRing * kStageVecs) + wv * (4 * kWave);
  auto raw_of = [&](int t) { return raw_base + (t & (kStages - 1)) * (kWgWaves * 4 * kWave); };
  auto request = [&](int32_t blk0, int32_t blk1, int t, bool again) {
    if (kFp8) request_tile_fp8(a, f, blk0, blk1, g, raw_of(t), again);
    else request_tile(a, f, blk0, blk1, g, stage_of(t), wv, again);
  };
  auto convert = [&](int t) {
    if (kFp8)
      convert_tile_fp8(lds_address(raw_of(t) + lane),
                       rd + ((t & (kRing - 1)) * kStageVecs + 2 * wv * kWave) * 16);
  };
  auto block_id = [&](int t, int which) { return sload(bt_row + min(2 * min(t, last) + which, n_blocks - 1)); };
  auto land = [&](int t) {  // after this wavefront's share of tile t arrived: mend a ragged tile
    const int n_valid = si.len - t * kTile;
    if (t <= last && n_valid < kTile) zero_invalid_v_lds(stage_of(t), wv, lane, n_valid);
  };

  __builtin_amdgcn_s_barrier();  // the previous segment is done with every stage
#pragma unroll
  for (int i = 0; i < kStages - 1; ++i)  // tiles t0 .. t0 + kStages - 2; past the end: the last tile again (L2 hits)
    request(block_id(t0 + i, 0), block_id(t0 + i, 1), t0 + i, t0 + i > last || si.rg > 1);
  int32_t nb0 = block_id(t0 + kStages - 1, 0), nb1 = block_id(t0 + kStages - 1, 1);
  asm volatile("" ::"s"(nb0), "s"(nb1));
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads * (kStages - 2)) : "memory");  // tile t0 is in
  convert(t0);
  land(t0);
  __builtin_amdgcn_s_barrier();
  floatx16 s;
  if (kRows) {
    score_tile(s, rd + (t0 & (kRing - 1)) * (kStageVecs * 16), q);
    if (si.len - t0 * kTile < kTile) mask_scores(s, si.len - t0 * kTile, h);
  }
  // iteration t: s_in holds the scores of tile t, s_out receives those of tile t + 1.  Only a sequence's last tile
  // can be ragged, so the iterations that land and mask a full tile (kChecked = false) carry no test for it.
  auto iter = [&](auto checked, int t, const floatx16& s_in, floatx16& s_out) {
    constexpr bool kChecked = decltype(checked)::value;
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(kLoads * (kStages - 3)) : "memory");  // tile t + 1 is in
    convert(t + 1);
    if (kChecked) land(t + 1);
    // every share of tile t + 1 is visible, and everyone is done with tile t - 1
    __builtin_amdgcn_s_barrier();
    auto fetch = [&]() {
      request(nb0, nb1, t + kStages - 1, t + kStages - 1 > last || si.rg > 1);
      nb0 = block_id(t + kStages, 0);
      nb1 = block_id(t + kStages, 1);
    };
    if (kRows) {
      const uint32_t k_addr = rd + ((t + 1) & (kRing - 1)) * (kStageVecs * 16);
      const uint32_t v_addr = rd + (t & (kRing - 1)) * (kStageVecs * 16) + 8 * kWave * 16;
      woven_tile(s_in, s_out, o, m, l, q, k_addr, v_addr, c, fetch);
      if (kChecked) {
        const int nv_next = si.len - (t + 1) * kTile;
        if (nv_next < kTile) mask_scores(s_out, nv_next, h);
      }
    } else {
      fetch();
    }
    // the block ids are in before the next iteration issues its LDS reads (no wait among them)
    asm volatile("" ::"s"(nb0), "s"(nb1));
  };
  // tile t + 1 is full for every t < len / kTile - 1
  const int t_plain = min(t1, si.len / kTile - 1);
  floatx16 s2;
  int t = t0;
  for (; t + 2 <= t_plain; t += 2) {
    iter(std::false_type{}, t, s, s2);
    iter(std::false_type{}, t + 1, s2, s);
  }
  for (; t < t1; ++t) {
    iter(std::true_type{}, t, s, s2);
    s = s2;
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no fetch of this segment may land later
  if (kRows) store_partial(slot, kLargeRows, wv, o, m, l, lane, a.m_scale, a.o_scale);
}

// One staged tile against this wavefront's 32 rows, nothing woven in: all 16 operand reads
// are issued up front, the counts of the waits follow that order.
__device__ inline void plain_tile(floatx16 (&o)[4], float& m, float& l, const bf16x8 (&q)[8], uint32_t k_addr,
                                  uint32_t v_addr, float c, int n_valid, int h) {
  bf16x8 kop[8], vop[8];
  lds_read_half(kop, k_addr, 0);
  lds_read_half(kop, k_addr, 1);
  lds_read_half(vop, v_addr, 0);
  lds_read_half(vop, v_addr, 1);
  floatx16 s = (floatx16)(0.f);
#define SMART_SCORE_STEP(I, N) \
  SMART_LDS_WAIT(kop[I], N);   \
  s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kop[I], q[I], s, 0, 0, 0);
  SMART_SCORE_STEP(0, 15)
  SMART_SCORE_STEP(1, 14)
  SMART_SCORE_STEP(2, 13)
  SMART_SCORE_STEP(3, 12)
  SMART_SCORE_STEP(4, 11)
  SMART_SCORE_STEP(5, 10)
  SMART_SCORE_STEP(6, 9)
  SMART_SCORE_STEP(7, 8)
#undef SMART_SCORE_STEP
  if (n_valid < kTile) mask_scores(s, n_valid, h);
  bf16x8 pb0, pb1;
  softmax_tile(s, m, l, o, pb0, pb1, c);
#define SMART_OUTPUT_STEP(I, N, PB) \
  SMART_LDS_WAIT(vop[I], N);        \
  o[I & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vop[I], PB, o[I & 3], 0, 0, 0);
  SMART_OUTPUT_STEP(0, 7, pb0)
  SMART_OUTPUT_STEP(1, 6, pb0)
  SMART_OUTPUT_STEP(2, 5, pb0)
  SMART_OUTPUT_STEP(3, 4, pb0)
  SMART_OUTPUT_STEP(4, 3, pb1)
  SMART_OUTPUT_STEP(5, 2, pb1)
  SMART_OUTPUT_STEP(6, 1, pb1)
  SMART_OUTPUT_STEP(7, 0, pb1)
#undef SMART_OUTPUT_STEP
}

// The states of a grouped segment (R row tiles x K = 8 / R key groups, wavefront = row tile *
// K + key group) become one partial: all eight states go to LDS, and after one barrier
// wavefront w merges, for row tile w / K, accumulator registers [(w % K) 64 / K, ...) of
// that row tile's K states (always in key-group order) and stores that slice.
template <int R>
__device__ inline void fold_groups(const SmallState& S, float* lds, float* slot, int rows_in_slot, int wv, int lane,
                                   float c) {
  constexpr int K = kWgWaves / R, kRegs = 64 / K;
  const int h = lane >> 5, j = lane & 31;
  state_to_lds(S, lds + wv * kStateFloats, lane);
  __syncthreads();
  const int rt = wv / K, part_index = wv % K;
  float mk[K], lk[K];
#pragma unroll
  for (int k = 0; k < K; ++k) {
    const float* src = lds + (rt * K + k) * kStateFloats;
    mk[k] = src[64 * kWave + lane];
    lk[k] = src[65 * kWave + lane];
  }
  floatx4 part[K][kRegs / 4];
#pragma unroll
  for (int k = 0; k < K; ++k)
#pragma unroll
    for (int u = 0; u < kRegs / 4; ++u)
      part[k][u] = state_quad(lds + (rt * K + k) * kStateFloats, part_index * (kRegs / 4) + u, lane);
  float m_new = mk[0];
#pragma unroll
  for (int k = 1; k < K; ++k) m_new = fmaxf(m_new, mk[k]);
  float l_new = 0.f;
  floatx4 x[kRegs / 4];
#pragma unroll
  for (int u = 0; u < kRegs / 4; ++u) x[u] = (floatx4)(0.f);
#pragma unroll
  for (int k = 0; k < K; ++k) {
    // an empty state has max -inf and contributes nothing
    const float sc = mk[k] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f((mk[k] - m_new) * c);
    l_new += lk[k] * sc;
#pragma unroll
    for (int u = 0; u < kRegs / 4; ++u) x[u] += part[k][u] * sc;
  }
  // accumulator register 16 jt + 4 r4 + i of lane (h, j) is row j, head dims 4 (8 jt + 2 r4 + h) + i
  const bool in_slot = rt * 32 < rows_in_slot;  // a 64-row slot has no room for row tiles 2 and 3 (they hold no rows)
#pragma unroll
  for (int u = 0; u < kRegs / 4; ++u) {
    const int reg = part_index * kRegs + 4 * u, jt = reg >> 4, r4 = (reg & 15) >> 2;
    if (in_slot) store_through(slot + ((size_t)(rt * 32 + jt * 8 + 2 * r4 + h) * 32 + j) * 4, x[u]);
  }
  if (part_index == 0) {
    const float lsum = sum_across_halves(l_new);
    if (h == 0 && in_slot) {
      slot[rows_in_slot * kD + rt * 32 + j] = m_new;
      slot[rows_in_slot * kD + rows_in_slot + rt * 32 + j] = lsum;
    }
  }
  __syncthreads();  // the next segment reuses the LDS
}

// Segments of at most 32 R rows (R = 2 or 4): the eight wavefronts are R row tiles x K = 8 / R
// key groups, and an iteration consumes K tiles at once (key group kg takes tile kg of the
// iteration), so that the stream, not the per-tile arithmetic of one wavefront, sets the pace.
// Tiles are staged as in staged_segment (every wavefront fetches an eighth of every tile); the
// iterations 8 / K - 1 ahead of the one being consumed are in flight.
template <int R>
__device__ inline void grouped_segment(const MainArgs& a, int b, int g, int base, int t0, int t1, const SeqInfo si,
                                       float* slot, int rows_in_slot, int wv, int lane, bf16x8* lds) {
  constexpr int K = kWgWaves / R;
  constexpr int kAhead = kStages / K - 1;
  // (row tile = wv / K: when only the first row tiles hold rows, the busy wavefronts sit on different SIMDs)
  const int rt = wv / K, kg = wv % K;
  const int h = lane >> 5, j = lane & 31;
  const int M = si.n * a.G;
  const bool has_rows = rt * 32 < M;
  SmallState S;
  bf16x8 q[8];
#pragma unroll
  for (int jt = 0; jt < 4; ++jt) S.o[jt] = (floatx16)(0.f);
  S.m = -INFINITY;
  S.l = 0.f;
  if (has_rows) {
    int rho = rt * 32 + j;
    rho = rho < M ? rho : M - 1;  // padding rows repeat the last real row; never read back
    const int node = base + rho / a.G, head = g * a.G + rho % a.G;
    const __bf16* qp = a.q + ((int64_t)node * a.Hq + head) * kD + h * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) q[ks] = *(const bf16x8*)(qp + ks * 16);
    asm volatile("" ::"v"(q[0]), "v"(q[7]));  // landed: the counted waits below see tile fetches only
  }
  const int32_t* bt_row = a.block_table + (int64_t)b * a.max_blocks;
  const int n_blocks = (si.len + kBlock - 1) / kBlock;
  const float c = a.scale_log2e;
  const FetchLane f = fetch_lane(a, wv, lane);
  const uint32_t rd = lds_address(lds + lane);
  const int last = t1 - 1;
  auto stage_of = [&](int t) { return lds + (t & (kStages - 1)) * kStageVecs; };
  auto block_id = [&](int t, int which) { return sload(bt_row + min(2 * min(t, last) + which, n_blocks - 1)); };
  auto land = [&](int t) {
    const int n_valid = si.len - t * kTile;
    if (t <= last && n_valid < kTile) zero_invalid_v_lds(stage_of(t), wv, lane, n_valid);
  };

  __builtin_amdgcn_s_barrier();  // the previous segment is done with the LDS
#pragma unroll
  for (int i = 0; i < kAhead * K; ++i)  // past the end: the last tile again (L2 hits), never consumed
    request_tile(a, f, block_id(t0 + i, 0), block_id(t0 + i, 1), g, stage_of(t0 + i), wv, t0 + i > last || si.rg > 1);
  int32_t nb[K][2];
#pragma unroll
  for (int x = 0; x < K; ++x) {
    nb[x][0] = block_id(t0 + kAhead * K + x, 0);
    nb[x][1] = block_id(t0 + kAhead * K + x, 1);
  }
  for (int tb = t0; tb < t1; tb += K) {
#pragma unroll
    for (int x = 0; x < K; ++x) asm volatile("" ::"s"(nb[x][0]), "s"(nb[x][1]));  // ids are in (no wait among LDS reads)
    // this wavefront's share of the K tiles of this iteration has landed: what may still be
    // outstanding are the kAhead - 1 iterations after it, 2 K fetches each
    if (K == 4) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
#pragma unroll
    for (int x = 0; x < K; ++x) land(tb + x);
    // every share of this iteration's tiles is visible, and everyone is done with the previous iteration's
    __builtin_amdgcn_s_barrier();
#pragma unroll
    for (int x = 0; x < K; ++x)
      request_tile(a, f, nb[x][0], nb[x][1], g, stage_of(tb + kAhead * K + x), wv, tb + kAhead * K + x > last || si.rg > 1);
#pragma unroll
    for (int x = 0; x < K; ++x) {
      nb[x][0] = block_id(tb + (kAhead + 1) * K + x, 0);
      nb[x][1] = block_id(tb + (kAhead + 1) * K + x, 1);
    }
    const int t = tb + kg;
    if (has_rows && t < t1) {
      const uint32_t stage = rd + (t & (kStages - 1)) * (kStageVecs * 16);
      plain_tile(S.o, S.m, S.l, q, stage, stage + 8 * kWave * 16, c, si.len - t * kTile, h);
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no fetch of this segment may land later
  __builtin_amdgcn_s_barrier();                      // and nobody still reads a stage: the fold reuses the LDS
  fold_groups<R>(S, (float*)lds, slot, rows_in_slot, wv, lane, c);
}

// Worker of classes 1 and 2 (kCls): a workgroup walks the pieces of its share of the class's units.
template <int kCls, bool kFp8 = false>
__device__ inline void staged_worker(const MainArgs& a, int64_t w, ClassPlan& cp, bf16x8* lds /* 132 KB: kStages tiles, or eight states */) {
  const PlanView pv = plan_view(a.plan, a.batch);
  const int64_t U = cp.U, W = cp.W;
  PlanWindow& win = cp.win;
  if (w >= W || U <= 0) return;
  int64_t u0 = share_begin(w, U, W);
  const int64_t u1 = share_begin(w + 1, U, W);
  if (u0 >= u1) return;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int b = locate(cp, pv, a.cu_nodes, kCls, a.batch, u0, lane);
  while (u0 < u1 && b < a.batch) {
    follow(cp, pv, a.cu_nodes, kCls, a.batch, b, lane);
    const int64_t seq_begin = window_cum_units(win, b - win.first);
    const int64_t seq_end = window_cum_units(win, b + 1 - win.first);
    if (u0 >= seq_end) { ++b; continue; }
    const SeqInfo si = window_info(win, b);
    const int64_t local = u0 - seq_begin;
    const int base = __builtin_amdgcn_readlane(win.cu_nodes, b - win.first);
    if (kCls == 1) {
      const int seg_local = (int)(local / si.tiles);
      const int t0 = (int)(local % si.tiles);
      const int g = seg_local;
      const int64_t left = u1 - u0;
      const int nt = (int)(left < (int64_t)(si.tiles - t0) ? left : (int64_t)(si.tiles - t0));
      const int64_t seg = (int64_t)__builtin_amdgcn_readlane(win.cum_segs, b - win.first) + seg_local;
      // At most 64 rows: row tiles 0 and 1 of four, times two key groups.  (Two row tiles x four
      // key groups would keep every wavefront busy but leaves only one iteration of fetches in
      // flight; measured slower.)
      grouped_segment<4>(a, b, g, base, t0, t0 + nt, si, a.ws[1] + (size_t)(w + seg) * kMediumSlot, kMediumRows, wv,
                         lane, lds);
      u0 += nt;
    } else {
      // the unit space of class 2 is a cost: see large_spans and large_tile_at
      const LargeSpans ls = large_spans(si, a.G);
      const int g = (int)(local / ls.span_head);
      const int64_t in_head = local - (int64_t)g * ls.span_head;
      int rgi = (int)(in_head / ls.span_full);
      rgi = rgi < si.rg - 1 ? rgi : si.rg - 1;
      const int64_t off = in_head - (int64_t)rgi * ls.span_full;
      const int cost = rgi < si.rg - 1 ? kLargeTileCost[kLargeRows / 32] : ls.cost_last;
      const int64_t span = rgi < si.rg - 1 ? ls.span_full : ls.span_last;
      const int seg_local = g * si.rg + rgi;
      const int64_t seg_end = u0 - off + span;
      const int64_t stop = u1 < seg_end ? u1 : seg_end;
      const int t0 = large_tile_at(off, cost, si.tiles);
      const int t1 = stop == seg_end ? si.tiles : large_tile_at(off + (stop - u0), cost, si.tiles);
      u0 = stop;
      const int64_t seg = (int64_t)__builtin_amdgcn_readlane(win.cum_segs, b - win.first) + seg_local;
      float* slot = a.ws[2] + (size_t)(w + seg) * kLargeSlot;
      if (t1 <= t0) {
        // The share covers less than a tile of this segment (rare).  The combine step
        // merges the partial of every worker whose share touches the segment, so this one leaves a partial that adds
        // nothing: row maxima of -inf (weight exp2(-inf) = 0), sums and O of zero.
        for (int i = threadIdx.x; i < kLargeSlot; i += kWgWaves * kWave)
          slot[i] = i >= kLargeRows * kD && i < kLargeRows * kD + kLargeRows ? -INFINITY : 0.f;
        continue;
      }
      // rows of the group are dealt to the eight wavefronts in 32-row tiles
      const int row0 = rgi * kLargeRows + wv * 32;
      if (row0 < si.n * a.G) staged_segment<true, kFp8>(a, b, g, base, row0, t0, t1, si, slot, wv, lane, lds);
      else staged_segment<false, kFp8>(a, b, g, base, row0, t0, t1, si, slot, wv, lane, lds);
    }
  }
}

// ---- the prefix kernel: one launch, workgroups apportioned to the classes by the plan ------
// kFp8: the cache holds E4M3 bytes; trees of up to 64 rows are class 1 and streamed into registers by
// fp8_worker, larger ones are class 2 and go through the staged loop after conversion to bf16 in LDS.
template <bool kFp8>
__global__ __launch_bounds__(kWgWaves * kWave) __attribute__((amdgpu_waves_per_eu(2, 2)))
void tva_prefix_kernel(MainArgs a) {
  __shared__ float4 lds_raw[8448];  // 132 KB, carved up per class (class 0: eight states of 16.5 KB)
  SMART_TIMELINE(const unsigned long long tl_start = wall_clock64(); const unsigned long long tl_cycles = clock64();)
  // Workgroups are dealt to the eight XCDs round robin; consecutive WORKERS (consecutive unit ranges: the row groups
  // of one segment, the two ends of a segment) are put on one XCD so that what they read in common meets in its L2.
  const int64_t wg = gridDim.x % 8 == 0 ? (int64_t)(blockIdx.x % 8) * (gridDim.x / 8) + blockIdx.x / 8 : (int64_t)blockIdx.x;
  const int lane = threadIdx.x & (kWave - 1);
  const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  ClassPlan cp;
  int64_t first1, first2, end;
  if (a.batch <= kWave) {
    // No planning kernel ran: wavefront 0 derives the plan and hands it to the others through
    // LDS; workgroup 0 also writes it to memory for the combine kernel.
    __shared__ PlanShare share;
    if (wv == 0) {
      LanePlan lp;
      lane_plan<kFp8>(lp, a.prefix_len, a.cu_nodes, a.batch, a.total_nodes, a.G, a.Hkv, a.max_blocks, a.workgroups, a.caps,
                      lane);
#pragma unroll
      for (int c = 0; c < kClasses; ++c) {
        share.cum_units[c][lane] = lp.cum_units[c];
        share.cum_segs[c][lane] = lp.cum_segs[c];
      }
      share.cu[lane] = lp.cu;
      share.info[lane] = lp.si;
      if (lane == 0) {
#pragma unroll
        for (int c = 0; c < kClasses; ++c) {
          share.units[c] = lp.units[c];
          share.workers[c] = lp.workers[c];
          share.first_wg[c] = lp.first_wg[c];
        }
        share.first_wg[kClasses] = lp.first_wg[kClasses];
      }
      if (wg == 0) {
        const PlanView pv = plan_view(a.plan, a.batch);
        if (lane <= a.batch) {
#pragma unroll
          for (int c = 0; c < kClasses; ++c) {
            pv.cum_units[c][lane] = lp.cum_units[c];
            pv.cum_segs[c][lane] = lp.cum_segs[c];
          }
          pv.cum_chunks[lane] = lp.cum_chunks;
        }
        if (a.batch == kWave && lane == 0) {  // entry 64 has no lane: the totals
#pragma unroll
          for (int c = 0; c < kClasses; ++c) {
            pv.cum_units[c][kWave] = lp.units[c];
            pv.cum_segs[c][kWave] = lp.total_segs[c];
          }
          pv.cum_chunks[kWave] = lp.chunks;
        }
        if (lane < a.batch) pv.info[lane] = lp.si;
        if (lane == 0) {
#pragma unroll
          for (int c = 0; c < kClasses; ++c) {
            pv.header[2 * c] = lp.units[c];
            pv.header[2 * c + 1] = lp.workers[c];
            pv.header[6 + c] = lp.first_wg[c];
          }
          pv.header[6 + kClasses] = lp.first_wg[kClasses];
        }
      }
    }
    __syncthreads();
    first1 = uniform64(share.first_wg[1]), first2 = uniform64(share.first_wg[2]), end = uniform64(share.first_wg[3]);
    const int cls = wg < first1 ? 0 : (wg < first2 ? 1 : 2);
    cp.U = uniform64(share.units[cls]);
    cp.W = uniform64(share.workers[cls]);
    cp.resident = true;
    cp.win.first = 0;
    cp.win.cum_units = share.cum_units[cls][lane];
    cp.win.cum_segs = share.cum_segs[cls][lane];
    cp.win.cu_nodes = share.cu[lane];
    const SeqInfo si = share.info[lane];
    cp.win.len = si.len;
    cp.win.n = si.n;
    cp.win.tiles = si.tiles;
    cp.win.rg = si.rg;
    cp.win.total_units = cp.U;
  } else {
    const PlanView pv = plan_view(a.plan, a.batch);
    first1 = sload(pv.header + 7), first2 = sload(pv.header + 8), end = sload(pv.header + 9);
    const int cls = wg < first1 ? 0 : (wg < first2 ? 1 : 2);
    cp.U = sload(pv.header + 2 * cls);
    cp.W = sload(pv.header + 2 * cls + 1);
    cp.resident = false;
  }
  if (wg >= end) return;
  SMART_TIMELINE(auto tl_end = [&]() {
    __syncthreads();  // the workgroup's end is its last wavefront's
    if (threadIdx.x == 0 && blockIdx.x < timeline::kWorkgroups) {
      unsigned long long* d = timeline::wg_stamps + 4 * blockIdx.x;
      d[0] = tl_start;
      d[1] = wall_clock64();
      d[2] = clock64() - tl_cycles;
      d[3] = (unsigned long long)(wg < first1 ? 0 : (wg < first2 ? 1 : 2)) | ((unsigned long long)wg << 8) | (1ull << 63);
    }
  };)
  if (kFp8) {
    if (wg >= first1 && wg < first2) fp8_worker(a, wg - first1, cp, (float*)lds_raw);
    else if (wg >= first2) staged_worker<2, true>(a, wg - first2, cp, (bf16x8*)lds_raw);
    SMART_TIMELINE(tl_end();)
    return;
  }
  if (wg < first1) {
    small_worker(a, wg, cp, (float*)lds_raw);
  } else if (wg < first2) {
    staged_worker<1>(a, wg - first1, cp, (bf16x8*)lds_raw);
  } else {
    staged_worker<2>(a, wg - first2, cp, (bf16x8*)lds_raw);
  }
  SMART_TIMELINE(tl_end();)
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
  const float* ws[kClasses];
  uint16_t* out;
  float* lse;
  int32_t batch, Hq, Hkv, G;
  float scale, scale_log2e;
  int32_t only_small;  // fp8 cache: the classes are those of plan_class<true>
  // block-table check (status may be null: no check)
  const int32_t* block_table;
  const int32_t* prefix_len;
  int32_t* status;
  int32_t max_blocks, num_blocks;
};

__device__ inline float bf16_to_f32(uint16_t x) { return __uint_as_float(((uint32_t)x) << 16); }
typedef __attribute__((ext_vector_type(2))) uint32_t uintx2;
typedef __attribute__((ext_vector_type(2))) float floatx2;
// A dword as a pair of bf16 values.  (The dword goes through a register of its own first: a bit cast applied
// directly to an element of a two-dword vector has been seen to read the vector's first element for both.)
__device__ inline bf16x2 bf16_pair(uint32_t w) {
  asm volatile("" : "+v"(w));
  return __builtin_bit_cast(bf16x2, w);
}
__device__ inline uint16_t f32_to_bf16(float v) {
  uint32_t u = __float_as_uint(v);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

// 8 lanes per query row; lane e of a row owns d = 4c .. 4c+3 for c = e, e+8, e+16, e+24.
// With one wavefront per SIMD (small batches of small trees) memory round trips are the cost here, so independent
// loads are issued together: the plan entries, the K and V rows of a step's tree keys, all of a partial's pieces.
// With several wavefronts per SIMD (large trees) the vector instructions of the tree part are, so it works on
// packed bf16 pairs (below), which also leaves room for five resident wavefronts per SIMD.
constexpr int kKeyPairs = 1;  // pairs of tree keys per step (2 and 4 measured slower: their registers cost resident wavefronts)

__global__ __launch_bounds__(kWave) void tva_combine_kernel(CombineArgs a) {
  const int wc = blockIdx.x;
  const int lane = threadIdx.x;
  SMART_TIMELINE(const unsigned long long tl_start = wall_clock64();)
  // the first `batch` wavefronts also check one sequence's block-table entries each (the grid has at least that many)
  if (a.status && wc < a.batch)
    smart::tva_validate_block_table(wc, a.block_table, a.prefix_len, a.max_blocks, kBlock, a.num_blocks, a.status, lane);
  const PlanView pv = plan_view(a.plan, a.batch);
  int b;
  if (a.batch <= kWave) {
    // cum_chunks is non-decreasing: lanes with cum <= wc are a prefix whose last lane is b
    const int32_t cum = pv.cum_chunks[min(lane, a.batch - 1)];
    const int32_t total = sload(pv.cum_chunks + a.batch);
    if (wc >= total) return;
    const uint64_t below = __ballot(lane < a.batch && cum <= wc);
    b = __popcll(below) - 1;
  } else {
    if (wc >= sload(pv.cum_chunks + a.batch)) return;
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
      const int mid = (lo + hi) >> 1;
      if (sload(pv.cum_chunks + mid) <= wc) lo = mid; else hi = mid;
    }
    b = lo;
  }
  const SeqInfo si = sload(pv.info + b);
  const int cls = a.only_small ? plan_class<true>(si.n * a.G) : seq_class(si.n * a.G);
  const int chunk_base = sload(pv.cum_chunks + b);
  const int base = sload(a.cu_nodes + b);
  const int64_t U = sload(pv.header + 2 * cls), W = sload(pv.header + 2 * cls + 1);
  // (selected with compares: indexing the pointer arrays with a run-time class would push the plan view to scratch)
  const int32_t* segs_c = cls == 0 ? pv.cum_segs[0] : (cls == 1 ? pv.cum_segs[1] : pv.cum_segs[2]);
  const int64_t* units_c = cls == 0 ? pv.cum_units[0] : (cls == 1 ? pv.cum_units[1] : pv.cum_units[2]);
  const int64_t seg_base = sload(segs_c + b);
  const int64_t unit_base = sload(units_c + b);
  const int M = si.n * a.G;
  const int per_g = (M + kCombineRows - 1) / kCombineRows;
  const int local = wc - chunk_base;
  const int g = local / per_g, chunk = local % per_g;
  const int e = lane & 7;
  const int rho_raw = chunk * kCombineRows + (lane >> 3);
  const bool active = rho_raw < M;
  const int rho = active ? rho_raw : M - 1;
  const int node = base + rho / a.G, head = g * a.G + rho % a.G;
  const float c = a.scale_log2e;

  // tree keys: the set bits of this row's ancestor mask, lowest first
  uint64_t mlo = active ? a.anc_mask[2 * (size_t)node] : 0ull;
  uint64_t mhi = active ? a.anc_mask[2 * (size_t)node + 1] : 0ull;
  uint32_t qw[8];  // the lane's 16 query elements as 8 bf16 pairs (dims 4 (e + 8 k) + 2 w, + 1)
  {
    const uint16_t* qp = a.q + ((int64_t)node * a.Hq + head) * kD;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const uintx2 x = *(const uintx2*)(qp + 4 * (e + 8 * k));
      qw[2 * k] = x[0];
      qw[2 * k + 1] = x[1];
    }
  }
  if (si.n < 64) mlo &= (1ull << si.n) - 1ull, mhi = 0ull;           // never index past the tree
  else if (si.n < 128) mhi &= (1ull << (si.n - 64)) - 1ull;

  float m = -INFINITY, l = 0.f, acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = 0.f;

  // Two keys per step, on the packed bf16 dot product: the score is q . k over bf16 pairs (products exact, sums in
  // binary32, as before); the two probabilities are rounded to bf16 like those of the matrix-core path, and one
  // instruction adds p0 v0[d] + p1 v1[d] to an output element (the V elements of the two keys paired by a byte
  // permute).  With several wavefronts per SIMD this loop is bound by its vector instructions, not by its loads.
  while (__any((mlo | mhi) != 0ull)) {
    int jn[2 * kKeyPairs];
    bool have[2 * kKeyPairs];
#pragma unroll
    for (int u = 0; u < 2 * kKeyPairs; ++u) {
      have[u] = (mlo | mhi) != 0ull;
      jn[u] = 0;
      if (mlo) { jn[u] = __ffsll((unsigned long long)mlo) - 1; mlo &= mlo - 1; }
      else if (mhi) { jn[u] = 64 + __ffsll((unsigned long long)mhi) - 1; mhi &= mhi - 1; }
    }
    uint32_t kw[2 * kKeyPairs][8], vw[2 * kKeyPairs][8];
#pragma unroll
    for (int u = 0; u < 2 * kKeyPairs; ++u) {
      const uint16_t* kp = a.k_tree + ((int64_t)(base + jn[u]) * a.Hkv + g) * kD;
      const uint16_t* vp = a.v_tree + ((int64_t)(base + jn[u]) * a.Hkv + g) * kD;
#pragma unroll
      for (int k = 0; k < 4; ++k) {
        const uintx2 x = *(const uintx2*)(kp + 4 * (e + 8 * k));
        const uintx2 y = *(const uintx2*)(vp + 4 * (e + 8 * k));
        kw[u][2 * k] = x[0];
        kw[u][2 * k + 1] = x[1];
        vw[u][2 * k] = y[0];
        vw[u][2 * k + 1] = y[1];
      }
    }
#pragma unroll
    for (int pr = 0; pr < kKeyPairs; ++pr) {
      float dot[2];
#pragma unroll
      for (int u = 0; u < 2; ++u) {
        float d0 = 0.f, d1 = 0.f;  // two chains
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
          d0 = __builtin_amdgcn_fdot2_f32_bf16(bf16_pair(qw[i]), bf16_pair(kw[2 * pr + u][i]), d0, false);
          d1 = __builtin_amdgcn_fdot2_f32_bf16(bf16_pair(qw[i + 1]), bf16_pair(kw[2 * pr + u][i + 1]), d1, false);
        }
        float d = d0 + d1;
        d += __shfl_xor(d, 1);
        d += __shfl_xor(d, 2);
        d += __shfl_xor(d, 4);
        dot[u] = have[2 * pr + u] ? d : -INFINITY;
      }
      const float m_new = fmaxf(m, fmaxf(dot[0], dot[1]));
      const float al = m_new == m ? 1.f : __builtin_amdgcn_exp2f((m - m_new) * c);  // (also when both are -inf)
      floatx2 p;
      p[0] = have[2 * pr] ? __builtin_amdgcn_exp2f((dot[0] - m_new) * c) : 0.f;
      p[1] = have[2 * pr + 1] ? __builtin_amdgcn_exp2f((dot[1] - m_new) * c) : 0.f;
      l = l * al + (p[0] + p[1]);
      m = m_new;
      const bf16x2 pp = __builtin_convertvector(p, bf16x2);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t lo = __builtin_amdgcn_perm(vw[2 * pr + 1][i], vw[2 * pr][i], 0x05040100u);  // (v0[d], v1[d])
        const uint32_t hi = __builtin_amdgcn_perm(vw[2 * pr + 1][i], vw[2 * pr][i], 0x07060302u);  // (v0[d + 1], v1[d + 1])
        acc[2 * i] = __builtin_amdgcn_fdot2_f32_bf16(bf16_pair(lo), pp, acc[2 * i] * al, false);
        acc[2 * i + 1] = __builtin_amdgcn_fdot2_f32_bf16(bf16_pair(hi), pp, acc[2 * i + 1] * al, false);
      }
    }
  }

  // prefix partials of this row's segment: workers w_first .. w_last of its class
  if (si.tiles > 0 && active) {
    const int rows_per_group = class_rows(cls);
    const int slot_floats = class_slot(cls);
    const float* ws = cls == 0 ? a.ws[0] : (cls == 1 ? a.ws[1] : a.ws[2]);
    const int rgi = rho / rows_per_group;
    const int seg_local = g * si.rg + rgi;
    const int64_t seg = seg_base + seg_local;
    const LargeSpans ls = large_spans(si, a.G);
    const bool last_group = rgi == si.rg - 1;
    const int64_t span = cls < 2 ? si.tiles : (last_group ? ls.span_last : ls.span_full);
    const int64_t ub = unit_base + (cls < 2 ? (int64_t)seg_local * si.tiles : g * ls.span_head + rgi * ls.span_full);
    const int64_t ue = ub + span - 1;
    const int64_t w_first = ((ub + 1) * W - 1) / U;
    const int64_t w_last = ((ue + 1) * W - 1) / U;
    const int row = rho % rows_per_group;  // = qt * 32 + j
    const int qt = row >> 5, j = row & 31;
    for (int64_t w = w_first; w <= w_last; ++w) {
      const float* slot = ws + (size_t)(w + seg) * slot_floats;
      const float mc = slot[rows_per_group * kD + row];
      const float lc = slot[rows_per_group * kD + rows_per_group + row];
      floatx4 x[4];
#pragma unroll
      for (int k = 0; k < 4; ++k)
        x[k] = *(const floatx4*)(slot + ((size_t)(qt * 32 + e + 8 * k) * 32 + j) * 4);
      const float m_new = fmaxf(m, mc);
      const float al = __builtin_amdgcn_exp2f((m - m_new) * c);
      const float wt = __builtin_amdgcn_exp2f((mc - m_new) * c);
      l = l * al + lc * wt;
#pragma unroll
      for (int k = 0; k < 4; ++k)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[4 * k + i] = acc[4 * k + i] * al + wt * x[k][i];
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
  SMART_TIMELINE(if (lane == 0 && wc < timeline::kWaves) {  // (lane 0's row always exists)
    timeline::wave_stamps[2 * wc] = tl_start;
    timeline::wave_stamps[2 * wc + 1] = wall_clock64();
  })
}

}  // namespace

namespace smart {

// Workgroups of the prefix kernel: one per compute unit (eight wavefronts, two per SIMD).  The
// plan deals them to the classes; a class never gets more workers than this bound.
static int32_t prefix_workgroups(const smart_ctx* ctx) {
  if (ctx->opt_workers > 0) return (int32_t)ctx->opt_workers;
  return ctx->num_cus > 0 ? ctx->num_cus : 256;
}
static int32_t class_workers(const smart_ctx* ctx, int cls) {
  const int32_t asked = prefix_workgroups(ctx);
  const int32_t wg = asked > kClasses ? asked : kClasses;
  (void)cls;
  return wg;  // a worker is a workgroup in every class
}
int32_t tva_mfma_default_workers(const smart_ctx* ctx) { return prefix_workgroups(ctx); }

// Segments per class a call can have at most when only the totals are known (every tree's size may be
// anything that adds up to total_nodes): one row group per sequence in classes 0 and 1; with an fp8
// cache every sequence is class 1, in row groups of 64 rows.
static void segment_bounds(int32_t batch, int32_t total_nodes, int32_t num_q_heads, int32_t num_kv_heads,
                           int64_t (&segs)[kClasses]) {
  const int64_t G = num_q_heads / num_kv_heads;
  segs[0] = (int64_t)num_kv_heads * batch;
  segs[1] = (int64_t)num_kv_heads * batch;
  segs[2] = (int64_t)num_kv_heads * (((int64_t)total_nodes * G + kLargeRows - 1) / kLargeRows + batch);
}

// The same from the trees' sizes (host copy of the offsets): exactly the segments the plan will count.
// False if the offsets are not a running sum inside [0, total_nodes].
static bool segment_counts(const int32_t* h_cu_nodes, int32_t batch, int32_t total_nodes, int32_t num_q_heads,
                           int32_t num_kv_heads, bool fp8, int64_t (&segs)[kClasses]) {
  const int G = num_q_heads / num_kv_heads;
  for (int c = 0; c < kClasses; ++c) segs[c] = 0;
  for (int32_t b = 0; b < batch; ++b) {
    const int64_t base = h_cu_nodes[b], next = h_cu_nodes[b + 1];
    if (base < 0 || next < base || next > total_nodes) return false;
    int64_t n = next - base;
    n = n > SMART_MAX_NODES ? SMART_MAX_NODES : n;
    const int rows = (int)n * G;
    if (rows == 0) continue;
    const int cls = fp8 ? plan_class<true>(rows) : seq_class(rows);
    if (cls < 2) segs[cls] += num_kv_heads;
    else segs[2] += (int64_t)num_kv_heads * ((rows + kLargeRows - 1) / kLargeRows);
  }
  return true;
}

// Slots of a class: worker w's piece of segment s goes to slot w + s.
static size_t class_slots(const smart_ctx* ctx, int cls, int64_t segs) {
  if (segs == 0) return 0;  // no sequence of this class: the plan gives it no worker
  return (size_t)class_workers(ctx, cls) + (size_t)segs + 1;
}

void tva_mfma_workspace(const smart_ctx* ctx, int32_t batch, int32_t total_nodes, int32_t num_q_heads,
                        int32_t num_kv_heads, size_t* ws_bytes, size_t* plan_bytes) {
  int64_t segs[kClasses];
  segment_bounds(batch, total_nodes, num_q_heads, num_kv_heads, segs);
  size_t floats = 0;
  for (int c = 0; c < kClasses; ++c) floats += class_slots(ctx, c, segs[c]) * class_slot(c);
  *ws_bytes = floats * sizeof(float);
  *plan_bytes = plan_bytes_for(batch);
}

bool tva_mfma_supported(const tva_params& p) {
  auto aligned16 = [](const void* x) { return ((uintptr_t)x & 15u) == 0; };
  return p.dtype == SMART_BF16 && p.kv_layout == SMART_KV_INTERLEAVED && p.head_dim == kD &&
         p.block_size == kBlock && p.cache_block_stride % 8 == 0 && p.cache_head_stride % 8 == 0 &&
         aligned16(p.d_q) && aligned16(p.d_k_cache) && aligned16(p.d_v_cache) &&
         aligned16(p.d_k_tree) && aligned16(p.d_v_tree) && aligned16(p.d_out) && p.num_blocks > 0;
}

int32_t tva_launch_mfma(smart_ctx* ctx, hipStream_t stream, const tva_params& p, const TvaWorkspace* fixed) {
  if (p.batch == 0 || p.total_nodes == 0) return SMART_OK;
  const int G = p.num_q_heads / p.num_kv_heads;
  const int32_t workgroups = prefix_workgroups(ctx);
  const bool fp8 = p.kv_cache_dtype == SMART_FP8_E4M3;
  // Room for partial results: by the totals alone (the context's own workspace, grown when needed), or, in a
  // caller-provided buffer of fixed size, by the trees' sizes when the host copy of the offsets is there.  The
  // plan counts the segments again on the device and runs nothing if they do not fit.
  SegCaps caps;
  if (!fixed || !p.h_cu_nodes) {
    segment_bounds(p.batch, p.total_nodes, p.num_q_heads, p.num_kv_heads, caps.segs);
  } else if (!segment_counts(p.h_cu_nodes, p.batch, p.total_nodes, p.num_q_heads, p.num_kv_heads, fp8, caps.segs)) {
    return SMART_EINVAL;
  }
  size_t slots[kClasses], floats = 0;
  for (int c = 0; c < kClasses; ++c) {
    slots[c] = class_slots(ctx, c, caps.segs[c]);
    floats += slots[c] * class_slot(c);
  }
  const size_t ws_bytes = floats * sizeof(float), plan_bytes = plan_bytes_for(p.batch);
  void* ws_base;
  void* plan_base;
  if (fixed) {
    if (ws_bytes > fixed->ws_bytes || plan_bytes > fixed->plan_bytes) return SMART_ECAP;
    ws_base = fixed->ws;
    plan_base = fixed->plan;
  } else {
    int32_t rc = ensure_workspace(ctx, stream, ws_bytes, plan_bytes);
    if (rc != SMART_OK) return rc;
    ws_base = ctx->ws;
    plan_base = ctx->plan;
  }
  float* ws[kClasses];
  ws[0] = (float*)ws_base;
  for (int c = 1; c < kClasses; ++c) ws[c] = ws[c - 1] + slots[c - 1] * class_slot(c - 1);

  if (p.batch > kWave) {  // smaller batches: the prefix kernel derives the plan itself
    if (fp8)
      hipLaunchKernelGGL(tva_plan_kernel<true>, dim3(1), dim3(kWave), 0, stream, plan_base, p.batch,
                         p.total_nodes, G, p.num_kv_heads, p.max_blocks_per_seq, workgroups, caps, p.d_prefix_len,
                         p.d_cu_nodes);
    else
      hipLaunchKernelGGL(tva_plan_kernel<false>, dim3(1), dim3(kWave), 0, stream, plan_base, p.batch,
                         p.total_nodes, G, p.num_kv_heads, p.max_blocks_per_seq, workgroups, caps, p.d_prefix_len,
                         p.d_cu_nodes);
    SMART_HIP_CHECK(hipGetLastError());
  }

  MainArgs ma;
  ma.q = (const __bf16*)p.d_q;
  ma.k_cache = (const __bf16*)p.d_k_cache;
  ma.v_cache = (const __bf16*)p.d_v_cache;
  ma.block_table = p.d_block_table;
  ma.cu_nodes = p.d_cu_nodes;
  ma.prefix_len = p.d_prefix_len;
  ma.total_nodes = p.total_nodes;
  ma.workgroups = workgroups;
  ma.plan = plan_base;
  ma.caps = caps;
  for (int c = 0; c < kClasses; ++c) ma.ws[c] = ws[c];
  ma.block_stride = p.cache_block_stride;
  ma.head_stride = p.cache_head_stride;
  ma.batch = p.batch;
  ma.Hq = p.num_q_heads;
  ma.Hkv = p.num_kv_heads;
  ma.G = G;
  ma.max_blocks = p.max_blocks_per_seq;
  ma.num_blocks = p.num_blocks;
  ma.scale_log2e = p.softmax_scale * kLog2e * (fp8 ? p.k_scale : 1.f);
  ma.m_scale = fp8 ? p.k_scale : 1.f;
  ma.o_scale = fp8 ? p.v_scale : 1.f;
  // (every class with work needs a workgroup, however few were asked for)
  const dim3 grid(workgroups > kClasses ? workgroups : kClasses);
  hipEvent_t ev_start = nullptr, ev_stop = nullptr;
  if (profile_events(ctx, &ev_start, &ev_stop)) {
    // a recorded call: the events ride on the dispatch and hold the kernel's own start and end
    if (fp8)
      hipExtLaunchKernelGGL(tva_prefix_kernel<true>, grid, dim3(kWgWaves * kWave), 0, stream, ev_start, ev_stop, 0, ma);
    else
      hipExtLaunchKernelGGL(tva_prefix_kernel<false>, grid, dim3(kWgWaves * kWave), 0, stream, ev_start, ev_stop, 0, ma);
    SMART_HIP_CHECK(hipGetLastError());
    profile_launched(ctx);
  } else {
    if (fp8)
      hipLaunchKernelGGL(tva_prefix_kernel<true>, grid, dim3(kWgWaves * kWave), 0, stream, ma);
    else
      hipLaunchKernelGGL(tva_prefix_kernel<false>, grid, dim3(kWgWaves * kWave), 0, stream, ma);
    SMART_HIP_CHECK(hipGetLastError());
  }

  CombineArgs ca;
  ca.q = (const uint16_t*)p.d_q;
  ca.k_tree = (const uint16_t*)p.d_k_tree;
  ca.v_tree = (const uint16_t*)p.d_v_tree;
  ca.cu_nodes = p.d_cu_nodes;
  ca.anc_mask = p.d_anc_mask;
  ca.plan = plan_base;
  for (int c = 0; c < kClasses; ++c) ca.ws[c] = ws[c];
  ca.out = (uint16_t*)p.d_out;
  ca.lse = p.d_lse;
  ca.batch = p.batch;
  ca.Hq = p.num_q_heads;
  ca.Hkv = p.num_kv_heads;
  ca.G = G;
  ca.scale = p.softmax_scale;
  ca.scale_log2e = p.softmax_scale * kLog2e;
  ca.only_small = fp8 ? 1 : 0;
  ca.block_table = p.d_block_table;
  ca.prefix_len = p.d_prefix_len;
  ca.status = p.d_status;
  ca.max_blocks = p.max_blocks_per_seq;
  ca.num_blocks = p.num_blocks;
  const int64_t max_chunks =
      (int64_t)p.num_kv_heads * (((int64_t)p.total_nodes * G + kCombineRows - 1) / kCombineRows + p.batch);
  if (max_chunks > 0x7FFFFFFF) return SMART_EINVAL;
  hipLaunchKernelGGL(tva_combine_kernel, dim3((unsigned)max_chunks), dim3(kWave), 0, stream, ca);
  SMART_HIP_CHECK(hipGetLastError());
  return SMART_OK;
}

}  // namespace smart

#ifdef SMART_TVA_TIMELINE
// Stamps of the last launch on the current device into host arrays of 4 x 1024 and 2 x 16384 words (unused entries
// are zero after smart_timeline_clear); both calls synchronize the device.
extern "C" int32_t smart_timeline_read(uint64_t* h_workgroups, uint64_t* h_waves) {
  if (!h_workgroups || !h_waves) return SMART_EINVAL;
  SMART_HIP_CHECK(hipDeviceSynchronize());
  SMART_HIP_CHECK(hipMemcpyFromSymbol(h_workgroups, HIP_SYMBOL(timeline::wg_stamps), sizeof(timeline::wg_stamps)));
  SMART_HIP_CHECK(hipMemcpyFromSymbol(h_waves, HIP_SYMBOL(timeline::wave_stamps), sizeof(timeline::wave_stamps)));
  return SMART_OK;
}
extern "C" int32_t smart_timeline_clear() {
  SMART_HIP_CHECK(hipDeviceSynchronize());
  void* p = nullptr;
  SMART_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(timeline::wg_stamps)));
  SMART_HIP_CHECK(hipMemset(p, 0, sizeof(timeline::wg_stamps)));
  SMART_HIP_CHECK(hipGetSymbolAddress(&p, HIP_SYMBOL(timeline::wave_stamps)));
  SMART_HIP_CHECK(hipMemset(p, 0, sizeof(timeline::wave_stamps)));
  return SMART_OK;
}
#endif
