// gs_sgns_step: one SGNS training iteration (GraphScale Sec. 3.2: fetch the
// rows the batch names, loss and sparse gradient on them, write them back, with
// the barrier of "Synchronization": all reads see the pre-iteration tables).
//
// The batch-synchronous rule is kept by splitting the iteration at kernel
// boundaries, and no atomic ever touches an embedding table: float atomics run
// at ~1/5 of the plain read-modify-write rate on this chip (and do not exist
// for a "round once" bf16 update), so contributions are first brought together
// per destination row and every touched row is written exactly once, as
// round(old + delta).
//
// Destination rows of both tables share one key space: key r < N is row r of
// the context table (its terms are the (pair, j) logits that name it), key N + c
// is row c of the input table (its terms are the staged gradients of the runs
// of equal centres).  A key has a counter slot: the key itself, or, when the
// graph is much larger than the batch, its place in a table of the batch's keys
// (so that nothing cleared, scanned or hit at random has the size of the graph).
//
//   clear      counters 0, key tables empty
//   forward    read-only on both tables: logits, g = dLoss/dx, loss, the
//              centre-row gradient of every run of equal centres staged in a
//              slot, and rank = cnt[slot of key]++ for every term and every
//              used staging slot (optionally the pairs themselves from the walk
//              buffer and the negatives from their counters)
//   scan       off = exclusive prefix sum of cnt
//   place      sorted[off[key] + rank] = (key, source row, coefficient, rank):
//              (context row, centre, -lr * g) or (N + centre, slot, -lr)
//   update     once over the context-table keys (source rows: the input table,
//              still unmodified), then once over the input-table keys (source
//              rows: the staged gradients): delta = sum coef * source row.  A
//              whole wave works on one row at a time.  The terms of a key are cut
//              into segments of 256 positions (64 in small batches); a row of one
//              segment is written once, as round(old + delta); the segments of a
//              longer row are added into a side buffer
//   finish     table[row] = round(old + side buffer) for the longer rows; one
//              extra block sums the per-block loss partials in a fixed order
//
// delta is accumulated exactly: every product coef * element is rounded once to
// a multiple of 2^-36 (one fp64 fused multiply-add against 1.5 * 2^52, whose
// result bits hold the integer) and the 64-bit integers are added.  Integer
// addition is associative, so the result does not depend on the order in which
// the terms of a row arrive (ranks come from atomics), on the places the keys
// get in their table, or on how a long row is split: the same call gives the
// same bits every time.
//
// Forward: a row is handled by 16 lanes holding 16-byte pieces (256 contiguous
// bytes per load instruction); a wave works on four rows at once and a dot
// product is a 16-lane DPP reduction.  No matrix cores: 0.3 flop per byte moved.
//
// The other entry points of this file run the same kernels with a few switches
// (SgnsArgs / SgnsExtras): the momentum and Adam steps write the row sums into
// the optimizer's tables between dense passes over whole tables; the fused step
// draws the negatives in the forward kernel; the one-table step (first-order
// LINE) reads the input rows in the update kernel from copies the forward kernel
// kept, because that kernel then writes rows of the table it would read.
#include <cmath>
#include <mutex>
#include <type_traits>

#include "common.h"

namespace gs {

constexpr int kSgnsThreads = 256;
constexpr int kGroupLanes = 16;
constexpr int kGroupsPerBlock = kSgnsThreads / kGroupLanes;
constexpr size_t kCompactFactor = 16;  // keys per batch entry beyond which the key space is compacted
constexpr int64_t kStageMaxBlocks = 8192;   // launch of the input-table pass (its waves stride over the slices)
constexpr int kStageSlice = 8;     // staged gradients per 16-lane group in the input-table pass: they are
                                   // few (one per run of equal centres), so short slices keep the chip busy
// Terms of one key are cut into segments of 2^seg_shift positions, each summed by one wave;
// rows with more than one segment go through the side buffer (slot = position of the row's
// first term >> seg_shift).  Long segments keep the side-buffer traffic low; small batches take
// short ones, so that the few waves of a launch do not wait for one that sums a long segment.
constexpr int kSegShiftLarge = 8, kSegShiftSmall = 6;
constexpr int kScanThreads = 256;
constexpr int kScanPerThread = 16;
constexpr int kScanTile = kScanThreads * kScanPerThread;
constexpr int64_t kFewTiles = 4096;   // up to this many scan tiles, blocks add up the earlier tile sums themselves
// Exact accumulation of the row sums: a product x = coef * element becomes the integer
// round(x * 2^36), read off the low bits of the fp64 value x * 2^36 + kFixMagic
// (one fused multiply-add; valid while |x| * 2^36 < 2^51, i.e. |x| < 32768).
constexpr double kFixScale = 68719476736.0;                  // 2^36
constexpr double kFixInvScale = 1.0 / 68719476736.0;
constexpr double kFixMagic = 6755399441055744.0;             // 1.5 * 2^52
constexpr unsigned long long kFixMagicBits = 0x4338000000000000ull;
constexpr float kFixPeak = 16384.0f;   // products at or beyond this magnitude are reported (NaN loss)
constexpr int kHotBits = 8;                      // block-local rank counters in forward
constexpr int kHotSlots = 1 << kHotBits;
constexpr uint32_t kRankPending = 0x80000000u;   // rank still relative to the block (ranks < 2^31)
constexpr uint32_t kNoRow = 0xffffffffu;         // no key: keys are below 2 * num_nodes <= 2^32 - 2


struct Term {      // one contribution to a destination row
  uint32_t row;    // key: context-table row r, or num_nodes + c for input-table row c
  int32_t center;  // source row: row of the input table (one-table mode: slot of its copy in
                   // `snap`), or the staging slot for an input-table key
  float coef;      // -lr * g, or -lr for a staged gradient
  uint32_t pos;    // position of this term among the terms of its key
};

struct SgnsArgs {
  void* w_in;               // tables the logits are computed from
  void* w_out;
  void* dst_in;             // tables that receive round(old + delta): the same two for plain
  void* dst_out;            // SGD, the momentum tables for the momentum step
  float* sq_in;             // Adam only (else null): with delta D of a row, the destination row
  float* sq_out;            // gets c1 * D and this second-moment row gets c2 * D * D (fp32 tables)
  float c1, c2;
  // negatives drawn inside the step (draw_negs != 0): entry (i, j) is the draw of
  // gs_sample_negatives for pair index neg_pair_base + i, written to negs_draw
  // (which `negs` then points to) for the later kernels
  int32_t draw_negs;
  const float* noise_prob;
  const int32_t* noise_alias;
  const uint2* noise_packed;
  uint64_t neg_seed;
  uint64_t neg_pair_base;
  int32_t* negs_draw;
  // pairs made inside the step (walks != null): pair i of the batch is pair first_pair + i of
  // the canonical pair sequence of walks[0 .. num_walks) (walk, then centre position, then
  // offset: the order of gs_make_pairs); pair_offsets[w] = number of pairs of the walks before
  // w, pair_offsets[num_walks] = all of them.  The forward kernel writes the ids it derives to
  // gen_centers / gen_contexts (which `centers` / `contexts` then point to) for the later kernels
  const int32_t* walks;
  const int64_t* pair_offsets;
  int64_t num_walks;
  int64_t first_pair;
  int32_t walk_len, window;
  int32_t* gen_centers;
  int32_t* gen_contexts;
  // one table on both sides (first-order LINE; else null): the update kernel writes rows of
  // the table while input rows are still needed, so the forward kernel keeps a copy of every
  // input row it loads (one per run of equal centres, at the run's staging slot) and notes
  // the slot of every pair; the update kernel reads the copies
  void* snap;               // [num_pairs][dim], storage type of the table
  int32_t* pair_slot;       // [num_pairs]
  const int32_t* centers;
  const int32_t* contexts;
  const int32_t* negs;
  int64_t num_pairs;
  int64_t num_nodes;
  int64_t num_terms;        // num_pairs * (k + 1): positions [0, num_terms) of `sorted` hold the
                            // context-table keys, the positions after them the input-table keys
  int64_t long_slots;       // ((num_terms + num_pairs) >> seg_shift) + 1
  int32_t seg_shift;        // log2 of the segment length
  int32_t chunk_pairs;      // consecutive pairs per 16-lane group in forward (<= 16)
  int32_t slice_terms;      // sorted terms per 16-lane group in update
  int32_t k;
  int32_t dim;
  float lr;
  float* g;                 // [num_terms]
  uint32_t* rank;           // [num_terms]
  uint32_t* cnt;            // [cnt_last + 1] counters, indexed by the slot of a key; after scan: offsets,
                            // and entry cnt_last holds the number of positions in use
  int64_t cnt_last;
  // Counter slots.  The context-table keys take the slots [0, in_base), the input-table keys
  // the slots from in_base on, so that in `sorted` every context-table key comes before every
  // input-table key.  A kind of key is either counted per vertex (bits == 0: slot = vertex) or,
  // when the graph is much larger than the batch, through an open-addressing table of
  // 1 << bits places holding the keys of the batch (slot = the key's place).  The batch has
  // few input-table keys (one per run of equal centres), so those go through a table sooner.
  uint32_t* key_table;      // [table_places = (out_bits ? 1 << out_bits : 0) + (in_bits ? 1 << in_bits : 0)],
                            // kNoRow = free
  int64_t table_places;
  int32_t out_bits, in_bits;
  uint32_t in_base;
  uint32_t* tile_sums;      // scan scratch
  Term* sorted;             // [num_terms + num_pairs]
  long long* long_acc;      // [long_slots][dim] exact sums of the long rows
  int32_t* stage_center;    // [num_pairs], -1 = unused slot
  uint32_t* stage_rank;     // [num_pairs] rank of the slot among the slots of its centre
  float* stage_delta;       // [num_pairs][dim], natural element order
  double* loss_partials;    // [forward blocks]
  int64_t forward_blocks;
  int64_t forward_blocks_per_xcd;
  double* loss_out;
  uint32_t* bad_ids;        // set when a centre / context / negative id is not a row of the tables,
                            // or a product left the range of the exact accumulation
};

// Ids come from device memory the host cannot inspect.  An id outside
// [0, num_nodes) is read as row 0 everywhere (so no access leaves the tables)
// and flagged; the call then reports a NaN loss.
__device__ __forceinline__ int32_t checked_row(const SgnsArgs& a, int32_t id) {
  if ((uint32_t)id < (uint32_t)a.num_nodes) return id;
  *a.bad_ids = 1u;
  return 0;
}

// ---- small device helpers ---------------------------------------------------------
// sum over the 16 lanes of a DPP row; every lane gets the total
__device__ __forceinline__ float row_sum16(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
  return x;
}

// every table type other than float is one of the 16-bit formats (bf16_t, f16_t)
template <typename T>
using if_16bit = std::enable_if_t<!std::is_same<T, float>::value, int>;

// Register image of a row: VPL float4 per lane.  Register v of lane l holds the
// elements [4q, 4q+4) with q = natural_q(v, l):
//   fp32 rows   one float4 per 16-byte load,  q = v*16 + l
//   16-bit rows two float4 per 16-byte load (8 elements), q = 2*((v/2)*16 + l) + (v&1)
template <typename T>
__device__ __forceinline__ int natural_q(int v, int l16) {
  return 2 * ((v >> 1) * kGroupLanes + l16) + (v & 1);
}
template <>
__device__ __forceinline__ int natural_q<float>(int v, int l16) { return v * kGroupLanes + l16; }

template <int VPL>
__device__ __forceinline__ void zero(float4 (&a)[VPL]) {
#pragma unroll
  for (int v = 0; v < VPL; ++v) a[v] = make_float4(0.f, 0.f, 0.f, 0.f);
}

template <int VPL>
__device__ __forceinline__ void load_row(const float* __restrict__ table, int64_t row, int dim,
                                         int l16, float4 (&r)[VPL]) {
  const float4* p = reinterpret_cast<const float4*>(table + row * (int64_t)dim);
  const int dim4 = dim >> 2;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int q = v * kGroupLanes + l16;
    r[v] = (q < dim4) ? p[q] : make_float4(0.f, 0.f, 0.f, 0.f);
  }
}

template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ void load_row(const T* __restrict__ table, int64_t row, int dim,
                                         int l16, float4 (&r)[VPL]) {
  static_assert(VPL % 2 == 0, "16-bit rows are held as pairs of float4");
  const uint4* p = reinterpret_cast<const uint4*>(table + row * (int64_t)dim);
  const int chunks = dim >> 3;
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w) {
    const int c = w * kGroupLanes + l16;
    if (c < chunks) {
      const uint4 x = p[c];
      r[2 * w] = make_float4(T::lo(x.x), T::hi(x.x), T::lo(x.y), T::hi(x.y));
      r[2 * w + 1] = make_float4(T::lo(x.z), T::hi(x.z), T::lo(x.w), T::hi(x.w));
    } else {
      r[2 * w] = make_float4(0.f, 0.f, 0.f, 0.f);
      r[2 * w + 1] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
  }
}

template <int VPL>
__device__ __forceinline__ float dot_partial(const float4 (&a)[VPL], const float4 (&b)[VPL]) {
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < VPL; ++v)
    s += a[v].x * b[v].x + a[v].y * b[v].y + a[v].z * b[v].z + a[v].w * b[v].w;
  return s;
}

template <int VPL>
__device__ __forceinline__ void axpy(float4 (&acc)[VPL], float c, const float4 (&x)[VPL]) {
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    acc[v].x += c * x[v].x; acc[v].y += c * x[v].y;
    acc[v].z += c * x[v].z; acc[v].w += c * x[v].w;
  }
}

// A row as it was loaded, kept in as few registers as its storage type needs:
// fp32 rows VPL float4, 16-bit rows VPL/2 uint4 (widened element by element where
// they are used).  Rows that wait in registers for their turn are held this way,
// so a 16-bit group keeps twice as many of them in flight.
template <typename T, int VPL>
struct RawRow { uint4 r[VPL / 2]; };
template <int VPL>
struct RawRow<float, VPL> { float4 r[VPL]; };

template <int VPL>
__device__ __forceinline__ void load_raw(const float* __restrict__ table, int64_t row, int dim, int l16,
                                         RawRow<float, VPL>& x) {
  load_row<VPL>(table, row, dim, l16, x.r);
}
template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ void load_raw(const T* __restrict__ table, int64_t row, int dim, int l16,
                                         RawRow<T, VPL>& x) {
  static_assert(VPL % 2 == 0, "16-bit rows are held as pairs of float4");
  const uint4* p = reinterpret_cast<const uint4*>(table + row * (int64_t)dim);
  const int chunks = dim >> 3;
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w) {
    const int c = w * kGroupLanes + l16;
    x.r[w] = (c < chunks) ? p[c] : make_uint4(0u, 0u, 0u, 0u);
  }
}

template <int VPL>
__device__ __forceinline__ void store_raw(float* __restrict__ table, int64_t row, int dim, int l16,
                                          const RawRow<float, VPL>& x) {
  float4* p = reinterpret_cast<float4*>(table + row * (int64_t)dim);
  const int dim4 = dim >> 2;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int q = v * kGroupLanes + l16;
    if (q < dim4) p[q] = x.r[v];
  }
}
template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ void store_raw(T* __restrict__ table, int64_t row, int dim, int l16,
                                          const RawRow<T, VPL>& x) {
  uint4* p = reinterpret_cast<uint4*>(table + row * (int64_t)dim);
  const int chunks = dim >> 3;
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w) {
    const int c = w * kGroupLanes + l16;
    if (c < chunks) p[c] = x.r[w];
  }
}

// Between two uses of a raw 16-bit row: makes the compiler widen it again at the
// second use instead of keeping the widened copy (twice the registers) alive.
template <int VPL>
__device__ __forceinline__ void rewiden_later(RawRow<float, VPL>&) {}
template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ void rewiden_later(RawRow<T, VPL>& x) {
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w)
    asm volatile("" : "+v"(x.r[w].x), "+v"(x.r[w].y), "+v"(x.r[w].z), "+v"(x.r[w].w));
}

template <int VPL>
__device__ __forceinline__ float dot_partial(const float4 (&a)[VPL], const RawRow<float, VPL>& b) {
  return dot_partial<VPL>(a, b.r);
}
template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ float dot_partial(const float4 (&a)[VPL], const RawRow<T, VPL>& b) {
  float s = 0.f;
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w) {
    const uint4 x = b.r[w];
    s += a[2 * w].x * T::lo(x.x) + a[2 * w].y * T::hi(x.x) + a[2 * w].z * T::lo(x.y) +
         a[2 * w].w * T::hi(x.y);
    s += a[2 * w + 1].x * T::lo(x.z) + a[2 * w + 1].y * T::hi(x.z) + a[2 * w + 1].z * T::lo(x.w) +
         a[2 * w + 1].w * T::hi(x.w);
  }
  return s;
}

template <int VPL>
__device__ __forceinline__ void axpy(float4 (&acc)[VPL], float c, const RawRow<float, VPL>& x) {
  axpy<VPL>(acc, c, x.r);
}
template <int VPL, typename T, if_16bit<T> = 0>
__device__ __forceinline__ void axpy(float4 (&acc)[VPL], float c, const RawRow<T, VPL>& b) {
#pragma unroll
  for (int w = 0; w < VPL / 2; ++w) {
    const uint4 x = b.r[w];
    acc[2 * w].x += c * T::lo(x.x); acc[2 * w].y += c * T::hi(x.x);
    acc[2 * w].z += c * T::lo(x.y); acc[2 * w].w += c * T::hi(x.y);
    acc[2 * w + 1].x += c * T::lo(x.z); acc[2 * w + 1].y += c * T::hi(x.z);
    acc[2 * w + 1].z += c * T::lo(x.w); acc[2 * w + 1].w += c * T::hi(x.w);
  }
}

// loss and dLoss/dx of one term from its logit: one expf, one log1pf, one divide
__device__ __forceinline__ void term_grad(float x, bool positive, float& g, float& loss) {
  const float e = expf(-fabsf(x));
  const float inv = 1.0f / (1.0f + e);
  const float sig = (x >= 0.0f) ? inv : e * inv;           // sigmoid(x)
  const float sig_m1 = (x >= 0.0f) ? -e * inv : -inv;      // sigmoid(x) - 1
  const float z = positive ? -x : x;
  loss = fmaxf(z, 0.0f) + log1pf(e);                       // softplus(z), |z| = |x|
  g = positive ? sig_m1 : sig;
}

// Blocks are handed to the 8 XCDs round-robin; this maps them so that each XCD
// works on one contiguous eighth of the batch: neighbouring chunks share
// centre and context rows, which then stay in that XCD's L2.  Performance only:
// any block-to-XCD assignment gives the same result.
__device__ __forceinline__ int64_t xcd_contiguous_block(int64_t bid, int64_t per_xcd) {
  return (bid & 7) * per_xcd + (bid >> 3);
}

// Counter slot of a key.  With the compacted key space the forward kernel enters the keys
// (claim_slot: first come, first served, linear probing; the table has at least twice as
// many places as the batch can hold keys) and the place kernel looks them up (find_slot).
// Which slot a key gets depends on the order of arrival, and with it the order of the rows in
// `sorted`; the results do not (exact sums).
struct KeyRegion {
  uint32_t slot_base;   // first counter slot of this kind of key
  uint32_t vertex;      // the key's vertex
  uint32_t* table;      // the kind's table (bits != 0)
  int bits;
};
__device__ __forceinline__ KeyRegion key_region(const SgnsArgs& a, uint32_t key) {
  const bool input_key = key >= (uint32_t)a.num_nodes;
  KeyRegion r;
  r.slot_base = input_key ? a.in_base : 0u;
  r.vertex = input_key ? key - (uint32_t)a.num_nodes : key;
  r.bits = input_key ? a.in_bits : a.out_bits;
  r.table = a.key_table + ((input_key && a.out_bits != 0) ? (1u << a.out_bits) : 0u);
  return r;
}
__device__ __forceinline__ uint32_t claim_slot(const SgnsArgs& a, uint32_t key) {
  const KeyRegion r = key_region(a, key);
  if (r.bits == 0) return r.slot_base + r.vertex;
  const uint32_t mask = (1u << r.bits) - 1u;
  const uint32_t home = (key * 2654435761u) >> (32 - r.bits);
  uint32_t h = home;
  // (the probe count is bounded so that the loop ends whatever the memory holds; a table
  // without a free place cannot arise from a batch the plan was made for, and is reported)
  for (uint32_t probes = 0; probes <= mask; ++probes) {
    uint32_t seen = __hip_atomic_load(r.table + h, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (seen == kNoRow) seen = atomicCAS(r.table + h, kNoRow, key);
    if (seen == kNoRow || seen == key) return r.slot_base + h;
    h = (h + 1u) & mask;
  }
  *a.bad_ids = 1u;
  return r.slot_base + home;
}
__device__ __forceinline__ uint32_t find_slot(const SgnsArgs& a, uint32_t key) {
  const KeyRegion r = key_region(a, key);
  if (r.bits == 0) return r.slot_base + r.vertex;
  const uint32_t mask = (1u << r.bits) - 1u;
  const uint32_t home = (key * 2654435761u) >> (32 - r.bits);
  uint32_t h = home;
  // every key of the batch was entered by the forward kernel
  for (uint32_t probes = 0; probes <= mask; ++probes) {
    if (r.table[h] == key) return r.slot_base + h;
    h = (h + 1u) & mask;
  }
  *a.bad_ids = 1u;
  return r.slot_base + home;
}

// ---- clear / fill ---------------------------------------------------------------------
// everything a call starts from: counters 0, no bad id seen (16 bytes per lane; the counter
// array is padded to a multiple of four entries)
__global__ void sgns_clear_kernel(uint4* __restrict__ cnt4, int64_t n4, uint4* __restrict__ table4,
                                  int64_t m4, uint32_t* __restrict__ flag) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i == 0) *flag = 0u;
  if (i < n4) cnt4[i] = make_uint4(0u, 0u, 0u, 0u);
  if (i < m4) table4[i] = make_uint4(kNoRow, kNoRow, kNoRow, kNoRow);
}

// ---- forward ------------------------------------------------------------------------------
// Staged centre-row gradient of one run of equal centres, in natural element
// order.  Slot numbers are fixed by position (first pair of the chunk + flush
// number), so no counter is shared between groups; unused slots of a chunk are
// marked with centre -1.
template <typename T, int VPL>
__device__ __forceinline__ void stage_flush(const SgnsArgs& a, int64_t slot, int32_t center, int l16,
                                            const float4 (&du)[VPL]) {
  if (l16 == 0) {
    a.stage_center[slot] = center;
    a.stage_rank[slot] = atomicAdd(a.cnt + claim_slot(a, (uint32_t)a.num_nodes + (uint32_t)center), 1u);
  }
  float4* out = reinterpret_cast<float4*>(a.stage_delta + slot * (int64_t)a.dim);
  const int dim4 = a.dim >> 2;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int q = natural_q<T>(v, l16);
    if (q < dim4) out[q] = du[v];
  }
}

// largest magnitude among the elements a lane holds of a row
template <int VPL>
__device__ __forceinline__ float row_peak(const float4 (&r)[VPL]) {
  float m = 0.f;
#pragma unroll
  for (int v = 0; v < VPL; ++v)
    m = fmaxf(fmaxf(m, fmaxf(fabsf(r[v].x), fabsf(r[v].y))), fmaxf(fabsf(r[v].z), fabsf(r[v].w)));
  return m;
}

template <typename T, int VPL, int RB>
__global__ __launch_bounds__(kSgnsThreads) void sgns_forward_kernel(SgnsArgs a) {
  extern __shared__ int32_t idx_s[];              // per group: centres[16], rows[16][K+1]
  __shared__ float loss_s[kGroupsPerBlock];
  // Rank counters of rows that many terms hit at once are same-address atomics in
  // memory, which serialise.  Each block therefore counts up to kHotSlots rows
  // locally first (whichever rows reach a slot of this small LDS table first):
  // a term of such a row takes a block-local rank, the block adds its total to
  // the row's global counter once, and the ranks are completed afterwards.
  __shared__ int32_t hot_key[kHotSlots];
  __shared__ uint32_t hot_cnt[kHotSlots];
  __shared__ uint32_t hot_base[kHotSlots];
  const T* __restrict__ w_in = static_cast<const T*>(a.w_in);
  const T* __restrict__ w_out = static_cast<const T*>(a.w_out);
  const int l16 = threadIdx.x & (kGroupLanes - 1);
  const int group_in_block = threadIdx.x / kGroupLanes;
  const int64_t block = xcd_contiguous_block(blockIdx.x, a.forward_blocks_per_xcd);
  const int K = a.k, K1 = a.k + 1;
  const int64_t group = block * kGroupsPerBlock + group_in_block;
  const int64_t first = group * a.chunk_pairs;
  const bool block_live = block < a.forward_blocks;
  const int64_t last = block_live ? min(first + a.chunk_pairs, a.num_pairs) : first;
  const int count = (int)max((int64_t)0, last - first);

  int32_t* cen_s = idx_s + group_in_block * (a.chunk_pairs * (K1 + 1));
  int32_t* rows_s = cen_s + a.chunk_pairs;
  for (int h = threadIdx.x; h < kHotSlots; h += kSgnsThreads) { hot_key[h] = -1; hot_cnt[h] = 0u; }
  if (a.walks != nullptr) {
    if (l16 < count) {                      // lane p derives pair p of the chunk from its walk
      int32_t c = 0, o = 0;
      const int64_t gp = a.first_pair + first + l16;
      if (gp < a.pair_offsets[a.num_walks]) {
        int64_t lo = 0, hi = a.num_walks - 1;     // last walk w with pair_offsets[w] <= gp
        while (lo < hi) {
          const int64_t mid = (lo + hi + 1) >> 1;
          if (a.pair_offsets[mid] <= gp) lo = mid; else hi = mid - 1;
        }
        const int32_t* row = a.walks + lo * (int64_t)a.walk_len;
        const int64_t len = valid_prefix(row, a.walk_len);
        int64_t at, other;
        pair_positions(gp - a.pair_offsets[lo], len, a.window, at, other);
        if (at >= 0 && at < len && other >= 0 && other < len) {
          c = row[at];
          o = row[other];
        } else {
          *a.bad_ids = 1u;                  // pair_offsets does not belong to these walks
        }
      } else {
        *a.bad_ids = 1u;                    // the walks do not hold that many pairs
      }
      a.gen_centers[first + l16] = c;
      a.gen_contexts[first + l16] = o;
      cen_s[l16] = checked_row(a, c);
      rows_s[l16 * K1] = checked_row(a, o);
    }
  } else if (l16 < count) {
    cen_s[l16] = checked_row(a, a.centers[first + l16]);
  }
  for (int t = l16; t < count * K1; t += kGroupLanes) {
    const int p = t / K1, j = t - p * K1;
    int32_t row;
    if (j == 0) {
      if (a.walks != nullptr) continue;     // set above
      row = checked_row(a, a.contexts[first + p]);
    } else if (a.draw_negs) {
      const Block4 b = philox_at(a.neg_seed, a.neg_pair_base + (uint64_t)(first + p), (uint32_t)(j - 1),
                                 0x80000000u);
      row = (int32_t)table_draw(a.noise_prob, a.noise_alias, a.noise_packed, (uint64_t)a.num_nodes, b);
      a.negs_draw[(first + p) * (int64_t)K + (j - 1)] = row;
    } else {
      row = checked_row(a, a.negs[(first + p) * (int64_t)K + (j - 1)]);
    }
    rows_s[t] = row;
  }
  __syncthreads();

  float4 u[VPL], du[VPL];
  zero<VPL>(u);
  zero<VPL>(du);
  int32_t cur_c = -1;
  int flushes = 0;
  float loss = 0.f;
  // The update kernels add products coef * element exactly while these stay below 32768:
  // coef is -lr * g with |g| <= 1 times an element of an input row, or -lr times an element
  // of a staged gradient.  Both kinds of rows pass through this kernel, which checks them.
  float peak = 0.f;

  for (int p = 0; p < count; ++p) {
    const int32_t c = cen_s[p];
    if (c != cur_c) {
      if (cur_c >= 0) {
        peak = fmaxf(peak, row_peak<VPL>(du));
        stage_flush<T, VPL>(a, first + flushes++, cur_c, l16, du);
      }
      load_row<VPL>(w_in, c, a.dim, l16, u);
      peak = fmaxf(peak, row_peak<VPL>(u));
      if (a.snap != nullptr) {              // one-table mode: keep the row as it is now
        RawRow<T, VPL> keep;
        load_raw<VPL>(w_in, c, a.dim, l16, keep);
        store_raw<VPL>(static_cast<T*>(a.snap), first + flushes, a.dim, l16, keep);
      }
      zero<VPL>(du);
      cur_c = c;
    }
    if (a.snap != nullptr && l16 == 0) a.pair_slot[first + p] = (int32_t)(first + flushes);
    const int64_t e0 = (first + p) * (int64_t)K1;
    const int32_t* prow = rows_s + p * K1;
    for (int j0 = 0; j0 <= K; j0 += RB) {
      // lane b of the group owns term j0 + b of this block of RB terms
      const int my_j = j0 + l16;
      const bool mine = l16 < RB && my_j <= K;
      uint32_t rk = 0;
      if (mine) {
        const int32_t row = prow[my_j];
        const uint32_t h = ((uint32_t)row * 2654435761u) >> (32 - kHotBits);
        const int32_t seen = atomicCAS(&hot_key[h], -1, row);
        if (seen == -1 || seen == row) rk = kRankPending | (atomicAdd(&hot_cnt[h], 1u) << kHotBits) | h;
        else rk = atomicAdd(a.cnt + claim_slot(a, (uint32_t)row), 1u);
      }
      RawRow<T, VPL> vv[RB];
#pragma unroll
      for (int b = 0; b < RB; ++b)
        if (j0 + b <= K) load_raw<VPL>(w_out, prow[j0 + b], a.dim, l16, vv[b]);
      float x_mine = 0.f;
#pragma unroll
      for (int b = 0; b < RB; ++b) {
        if (j0 + b <= K) {
          const float x = row_sum16(dot_partial<VPL>(u, vv[b]));
          if (l16 == b) x_mine = x;
        }
      }
#pragma unroll
      for (int b = 0; b < RB; ++b) rewiden_later<VPL>(vv[b]);
      float g_mine = 0.f, l_mine = 0.f;
      if (mine) term_grad(x_mine, my_j == 0, g_mine, l_mine);
      loss += l_mine;
#pragma unroll
      for (int b = 0; b < RB; ++b)
        if (j0 + b <= K) axpy<VPL>(du, __shfl(g_mine, b, kGroupLanes), vv[b]);
      if (mine) { a.g[e0 + my_j] = g_mine; a.rank[e0 + my_j] = rk; }
    }
  }
  if (cur_c >= 0) {
    peak = fmaxf(peak, row_peak<VPL>(du));
    stage_flush<T, VPL>(a, first + flushes++, cur_c, l16, du);
  }
  if (l16 >= flushes && l16 < count) a.stage_center[first + l16] = -1;
  if (!(peak * fabsf(a.lr) < kFixPeak)) *a.bad_ids = 1u;   // (also taken for NaN)

  loss = row_sum16(loss);
  if (l16 == 0) loss_s[group_in_block] = loss;
  __syncthreads();
  // one global update per locally counted row, then complete the pending ranks
  for (int h = threadIdx.x; h < kHotSlots; h += kSgnsThreads)
    if (hot_key[h] >= 0) hot_base[h] = atomicAdd(a.cnt + claim_slot(a, (uint32_t)hot_key[h]), hot_cnt[h]);
  __syncthreads();
  for (int t = l16; t < count * K1; t += kGroupLanes) {
    const int64_t e = first * (int64_t)K1 + t;
    // written above by another lane of this group: read it back past the L1
    const uint32_t rk = __hip_atomic_load(a.rank + e, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (rk & kRankPending)
      a.rank[e] = hot_base[rk & (kHotSlots - 1)] + ((rk & ~kRankPending) >> kHotBits);
  }
  if (threadIdx.x == 0 && block_live) {
    double s = 0.0;
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerBlock; ++gidx) s += (double)loss_s[gidx];
    a.loss_partials[block] = s;
  }
}

// ---- exclusive scan of cnt[0..n) (uint32), three kernels ---------------------
__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const uint32_t* __restrict__ data,
                                                                   int64_t n,
                                                                   uint32_t* __restrict__ tile_sums) {
  __shared__ uint32_t s[kScanThreads / 64];
  const int64_t base = (int64_t)blockIdx.x * kScanTile;
  uint32_t acc = 0;
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) {
    const int64_t i = base + (int64_t)k * kScanThreads + threadIdx.x;
    if (i < n) acc += data[i];
  }
#pragma unroll
  for (int d = 32; d > 0; d >>= 1) acc += __shfl_xor(acc, d, 64);
  if ((threadIdx.x & 63) == 0) s[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) t += s[w];
    tile_sums[blockIdx.x] = t;
  }
}

// single block: exclusive scan of the tile sums in place
__global__ __launch_bounds__(1024) void scan_tiles_kernel(uint32_t* __restrict__ tile_sums,
                                                          int64_t tiles) {
  __shared__ uint32_t wave_tot[16];
  __shared__ uint32_t carry_s;
  if (threadIdx.x == 0) carry_s = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int64_t base = 0; base < tiles; base += 1024) {
    const int64_t i = base + threadIdx.x;
    const uint32_t v = (i < tiles) ? tile_sums[i] : 0u;
    uint32_t incl = v;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const uint32_t up = __shfl_up(incl, d, 64);
      if (lane >= d) incl += up;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = carry_s, all = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
      if (w < wave) before += wave_tot[w];
      all += wave_tot[w];
    }
    if (i < tiles) tile_sums[i] = before + incl - v;
    __syncthreads();
    if (threadIdx.x == 0) carry_s += all;
    __syncthreads();
  }
}

// tile_offsets: exclusive prefix sums of the tile sums (raw_sums == 0), or the tile sums
// themselves (raw_sums != 0: each block adds up the sums of the tiles before it, which is
// cheaper than a kernel of its own while there are few tiles)
__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(uint32_t* __restrict__ data, int64_t n,
                                                                  const uint32_t* __restrict__ tile_offsets,
                                                                  int raw_sums) {
  __shared__ uint32_t wave_tot[kScanThreads / 64];
  __shared__ uint32_t before_s[kScanThreads / 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint32_t tile_base;
  if (raw_sums) {
    uint32_t part = 0;
    for (int64_t i = threadIdx.x; i < (int64_t)blockIdx.x; i += kScanThreads) part += tile_offsets[i];
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) part += __shfl_xor(part, d, 64);
    if (lane == 0) before_s[wave] = part;
    __syncthreads();
    tile_base = 0;
#pragma unroll
    for (int w = 0; w < kScanThreads / 64; ++w) tile_base += before_s[w];
  } else {
    tile_base = tile_offsets[blockIdx.x];
  }
  // thread t owns kScanPerThread consecutive values
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanPerThread;
  uint32_t v[kScanPerThread];
  uint32_t local = 0;
  const bool whole = base + kScanPerThread <= n;   // 64 aligned bytes: four 16-byte accesses
  if (whole) {
    const uint4* p4 = reinterpret_cast<const uint4*>(data + base);
#pragma unroll
    for (int k4 = 0; k4 < kScanPerThread / 4; ++k4) {
      const uint4 x = p4[k4];
      v[4 * k4] = x.x; v[4 * k4 + 1] = x.y;
      v[4 * k4 + 2] = x.z; v[4 * k4 + 3] = x.w;
    }
  } else {
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) v[k] = (base + k < n) ? data[base + k] : 0u;
  }
#pragma unroll
  for (int k = 0; k < kScanPerThread; ++k) local += v[k];
  uint32_t incl = local;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t run = tile_base + incl - local;
#pragma unroll
  for (int w = 0; w < kScanThreads / 64; ++w)
    if (w < wave) run += wave_tot[w];
  if (whole) {
    uint4* p4 = reinterpret_cast<uint4*>(data + base);
#pragma unroll
    for (int k4 = 0; k4 < kScanPerThread / 4; ++k4) {
      uint4 x;
      x.x = run; run += v[4 * k4];
      x.y = run; run += v[4 * k4 + 1];
      x.z = run; run += v[4 * k4 + 2];
      x.w = run; run += v[4 * k4 + 3];
      p4[k4] = x;
    }
  } else {
#pragma unroll
    for (int k = 0; k < kScanPerThread; ++k) {
      if (base + k < n) data[base + k] = run;
      run += v[k];
    }
  }
}

// The whole scan in one block, for the few counters of a small batch (one kernel instead of
// two on a path that is bound by its number of dependent kernels): a thread sums its stretch
// of consecutive entries, the block scans the sums, the thread writes its stretch.  Entries
// move 16 bytes at a time, eight independent loads in flight per thread: `data` is 16-byte
// aligned and allocated up to a multiple of four entries; the padding is read (it holds
// zeros) and written.
constexpr int64_t kScanSmallMax = 1 << 17;
__global__ __launch_bounds__(1024) void scan_small_kernel(uint32_t* __restrict__ data, int64_t n) {
  __shared__ uint32_t wave_tot[16];
  constexpr int kBurst = 8;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  uint4* __restrict__ d4 = (uint4*)data;
  const int64_t n4 = (n + 3) / 4;
  const int per = (int)((n4 + 1023) / 1024);
  const int64_t lo = min(n4, (int64_t)threadIdx.x * per);
  const int mine = (int)(min(n4, lo + per) - lo);
  uint32_t local = 0;
  for (int c = 0; c < mine; c += kBurst) {
    uint4 v[kBurst];
#pragma unroll
    for (int u = 0; u < kBurst; ++u) v[u] = (c + u < mine) ? d4[lo + c + u] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < kBurst; ++u) local += v[u].x + v[u].y + v[u].z + v[u].w;
  }
  uint32_t incl = local;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    const uint32_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  if (lane == 63) wave_tot[wave] = incl;
  __syncthreads();
  uint32_t run = incl - local;
#pragma unroll
  for (int w = 0; w < 16; ++w)
    if (w < wave) run += wave_tot[w];
  for (int c = 0; c < mine; c += kBurst) {
    uint4 v[kBurst];
#pragma unroll
    for (int u = 0; u < kBurst; ++u) v[u] = (c + u < mine) ? d4[lo + c + u] : make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int u = 0; u < kBurst; ++u) {
      uint4 o;
      o.x = run;
      o.y = o.x + v[u].x;
      o.z = o.y + v[u].y;
      o.w = o.z + v[u].z;
      run = o.w + v[u].w;
      if (c + u < mine) d4[lo + c + u] = o;
    }
  }
}

// ---- place: scatter the terms into key-major order ------------------------------
// Entries [0, num_terms) are the (pair, j) terms, entries num_terms + s the staging slots.
// The entry with position 2^seg_shift (it exists exactly in the rows of more than one
// segment) also clears the row's slot of the side buffer.
__global__ __launch_bounds__(256) void sgns_place_kernel(SgnsArgs a) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= a.num_terms + a.num_pairs) return;
  Term t;
  uint32_t rk;
  if (e < a.num_terms) {
    const int K1 = a.k + 1;
    const int64_t i = e / K1;
    const int j = (int)(e - i * K1);
    t.row = (uint32_t)checked_row(a, (j == 0) ? a.contexts[i] : a.negs[i * (int64_t)a.k + (j - 1)]);
    t.center = (a.pair_slot != nullptr) ? a.pair_slot[i] : checked_row(a, a.centers[i]);
    t.coef = -a.lr * a.g[e];
    rk = a.rank[e];
  } else {
    const int64_t slot = e - a.num_terms;
    const int32_t c = a.stage_center[slot];
    if (c < 0) return;
    t.row = (uint32_t)a.num_nodes + (uint32_t)c;
    t.center = (int32_t)slot;
    t.coef = -a.lr;
    rk = a.stage_rank[slot];
  }
  const uint32_t begin = a.cnt[find_slot(a, t.row)];
  t.pos = rk;
  a.sorted[begin + rk] = t;
  if (rk == (1u << a.seg_shift)) {
    long long* acc = a.long_acc + (int64_t)(begin >> a.seg_shift) * a.dim;
    for (int x = 0; x < a.dim; ++x) acc[x] = 0;
  }
}

// ---- update: one pass over the key-major terms of one table ----------------------------
// Here a whole wave works on one row at a time: the fields of a term are broadcast
// from the lane that holds it into scalar registers, so every branch (row change,
// long row, end of slice) is uniform and the per-row epilogue runs once per row.
// Lane l holds, for p < PPL, piece p*64 + l of a row; a piece is WPP 32-bit words of the
// table's storage type (4, 8 or 16 bytes: 256, 512 or 1024 contiguous bytes per load
// instruction), i.e. EPP = WPP (fp32) or 2 * WPP (16-bit) consecutive elements.
//
// Exact row sums: acc holds the sum of the result bits of fma(element, coef * 2^36,
// kFixMagic), i.e. terms * kFixMagicBits + the sum of the rounded products (mod 2^64).
__device__ __forceinline__ void fix_add(unsigned long long& acc, double c, float x) {
  acc += (unsigned long long)__double_as_longlong(__builtin_fma((double)x, c, kFixMagic));
}

template <typename T>
struct Words { static constexpr int kPerWord = 2; };     // elements in a 32-bit word of a table
template <>
struct Words<float> { static constexpr int kPerWord = 1; };

// one piece of WORDS 32-bit words, in a single load / store instruction
template <int WORDS>
__device__ __forceinline__ void load_words(const uint32_t* __restrict__ p, uint32_t (&w)[WORDS]) {
  if constexpr (WORDS == 1) {
    w[0] = *p;
  } else if constexpr (WORDS == 2) {
    const uint2 x = *reinterpret_cast<const uint2*>(p);
    w[0] = x.x; w[1] = x.y;
  } else {
    static_assert(WORDS % 4 == 0, "pieces are 4, 8 or a multiple of 16 bytes");
#pragma unroll
    for (int i = 0; i < WORDS / 4; ++i) {
      const uint4 x = reinterpret_cast<const uint4*>(p)[i];
      w[4 * i] = x.x; w[4 * i + 1] = x.y; w[4 * i + 2] = x.z; w[4 * i + 3] = x.w;
    }
  }
}
template <int WORDS>
__device__ __forceinline__ void store_words(uint32_t* __restrict__ p, const uint32_t (&w)[WORDS]) {
  if constexpr (WORDS == 1) {
    *p = w[0];
  } else if constexpr (WORDS == 2) {
    *reinterpret_cast<uint2*>(p) = make_uint2(w[0], w[1]);
  } else {
#pragma unroll
    for (int i = 0; i < WORDS / 4; ++i)
      reinterpret_cast<uint4*>(p)[i] = make_uint4(w[4 * i], w[4 * i + 1], w[4 * i + 2], w[4 * i + 3]);
  }
}

// element i of a piece held as words of storage type T, widened exactly
template <typename T, int WORDS>
__device__ __forceinline__ float piece_elem(const uint32_t (&w)[WORDS], int i) {
  if constexpr (std::is_same<T, float>::value) return __uint_as_float(w[i]);
  else return (i & 1) ? T::hi(w[i >> 1]) : T::lo(w[i >> 1]);
}

// the exact sum as a double: net integer (terms * magic bits taken off) times 2^-36
__device__ __forceinline__ double fix_value(unsigned long long acc) {
  return (double)(long long)acc * kFixInvScale;
}

__device__ __forceinline__ uint32_t uniform_u32(uint32_t x) {
  return (uint32_t)__builtin_amdgcn_readfirstlane((int)x);
}

// first position >= p (and < limit) whose term starts a segment, else limit; wave-uniform
__device__ __forceinline__ int64_t next_segment_start(const Term* __restrict__ sorted, int64_t p,
                                                      int64_t limit, int lane, uint32_t seg_mask) {
  while (p < limit) {
    const bool start = p + lane >= limit || (sorted[p + lane].pos & seg_mask) == 0u;
    const unsigned long long mask = __builtin_amdgcn_ballot_w64(start);
    if (mask != 0ull) return min(limit, p + (int64_t)__builtin_ctzll(mask));
    p += 64;
  }
  return limit;
}

// Ownership: the terms of a key are cut into segments of S = 2^seg_shift consecutive
// positions (pos = 0..S-1, S..2S-1, ...); a wave handles the segments whose first term lies
// in its slice, reading on past the slice's end to finish the last one.  A row of at most S
// terms is one segment: it is written once, as round(old + sum).  The partial sums of a row
// with more segments meet in the side buffer at slot (position of the row's first term) >>
// seg_shift, which no two such rows can share because each spans more than S positions.
// kStage = false: context-table keys, positions [0, num_terms), source rows from the input
// table; kStage = true: input-table keys, the positions after them, source rows = staged
// gradients (fp32, natural element order).
template <typename T, int WPP, int PPL, int UB, bool kSq, bool kStage>
__global__ __launch_bounds__(kSgnsThreads) void sgns_update_kernel(SgnsArgs a) {
  static_assert(!kSq || std::is_same<T, float>::value, "second-moment tables are fp32");
  constexpr int kWaves = kSgnsThreads / 64;
  constexpr int EPP = WPP * Words<T>::kPerWord;          // elements per piece
  constexpr int EPL = EPP * PPL;                         // elements per lane
  constexpr int SW = kStage ? EPP : WPP;                 // 32-bit words of a source piece
  // source rows: the input table, or the copies the forward kernel kept (one-table mode),
  // or the staged gradients
  const uint32_t* __restrict__ src_base = reinterpret_cast<const uint32_t*>(
      kStage ? static_cast<const void*>(a.stage_delta) : (a.snap != nullptr ? a.snap : a.w_in));
  uint32_t* dst_base = reinterpret_cast<uint32_t*>(kStage ? a.dst_in : a.dst_out);
  uint32_t* sq_base = reinterpret_cast<uint32_t*>(kStage ? a.sq_in : a.sq_out);
  const uint32_t key_base = kStage ? (uint32_t)a.num_nodes : 0u;
  const int64_t pos_lo = kStage ? a.num_terms : 0;
  // (scalars that come out of memory are made wave-uniform explicitly: loop bounds and the
  // lane numbers of the broadcasts below must live in scalar registers)
  const int64_t pos_hi = kStage ? (int64_t)uniform_u32(a.cnt[a.cnt_last]) : a.num_terms;
  const int lane = threadIdx.x & 63;
  const int64_t first_wave = (int64_t)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int slice = kStage ? kStageSlice : a.slice_terms;
  const Term* __restrict__ sorted = a.sorted;
  const int64_t src_row_words = kStage ? (int64_t)a.dim : (int64_t)a.dim / Words<T>::kPerWord;
  const int64_t dst_row_words = (int64_t)a.dim / Words<T>::kPerWord;
  bool piece_ok[PPL];                                    // piece p of this lane lies inside the row
#pragma unroll
  for (int p = 0; p < PPL; ++p) piece_ok[p] = (p * 64 + lane) * EPP < a.dim;

  const uint32_t seg_mask = (1u << a.seg_shift) - 1u;
  // a wave takes the slices first_wave, first_wave + (waves of the launch), ...: the launch of
  // the input-table pass is sized for the few slots a batch normally uses, not for one per pair
  for (int64_t wave = first_wave;; wave += (int64_t)gridDim.x * kWaves) {
  const int64_t slice_begin = pos_lo + wave * slice;
  if (slice_begin >= pos_hi) break;
  const int64_t slice_end = min(slice_begin + slice, pos_hi);
  const int64_t begin = next_segment_start(sorted, slice_begin, pos_hi, lane, seg_mask);   // what lies before is an earlier wave's
  const int64_t end = next_segment_start(sorted, slice_end, pos_hi, lane, seg_mask);       // finish the segment we started

  unsigned long long acc[EPL];
  uint32_t old[PPL][WPP];
#pragma unroll
  for (int x = 0; x < EPL; ++x) acc[x] = 0;
#pragma unroll
  for (int p = 0; p < PPL; ++p)
#pragma unroll
    for (int w = 0; w < WPP; ++w) old[p][w] = 0u;
  uint32_t cur_row = kNoRow;       // key of the segment being summed (table row: cur_row - key_base)
  uint32_t cur_seg = 0;            // its number within the key (pos >> seg_shift of its terms)
  int64_t seg_first = 0;           // position of its first term
  uint32_t cur_terms = 0;          // terms added into acc since it was cleared

  // takes the magic bits of the terms off (their low word is zero): acc becomes the net sum
  auto settle = [&]() {
    const unsigned long long off = (unsigned long long)(cur_terms * (uint32_t)(kFixMagicBits >> 32)) << 32;
#pragma unroll
    for (int x = 0; x < EPL; ++x) acc[x] -= off;
  };
  auto flush_long = [&]() {
    const int64_t row_first = seg_first - ((int64_t)cur_seg << a.seg_shift);
    unsigned long long* dst = reinterpret_cast<unsigned long long*>(a.long_acc) +
                              (row_first >> a.seg_shift) * a.dim;
#pragma unroll
    for (int p = 0; p < PPL; ++p) {
      if (piece_ok[p]) {
#pragma unroll
        for (int i = 0; i < EPP; ++i) atomicAdd(dst + (p * 64 + lane) * EPP + i, acc[p * EPP + i]);
      }
    }
  };
  // new = round(old + d) for the elements of one piece, packed back into storage words
  auto write_piece = [&](uint32_t* row_words, int p, const uint32_t (&was)[WPP], const double* d) {
    uint32_t out[WPP];
    if constexpr (std::is_same<T, float>::value) {
#pragma unroll
      for (int i = 0; i < WPP; ++i)
        out[i] = __float_as_uint((float)((double)__uint_as_float(was[i]) + d[i]));
    } else {
#pragma unroll
      for (int i = 0; i < WPP; ++i)
        out[i] = pack16<T>((float)((double)T::lo(was[i]) + d[2 * i]),
                           (float)((double)T::hi(was[i]) + d[2 * i + 1]));
    }
    store_words<WPP>(row_words + (int64_t)(p * 64 + lane) * WPP, out);
  };
  // continues: the next term belongs to the same key (the row has a further segment)
  auto flush = [&](bool continues) {
    settle();
    if (cur_seg > 0 || continues) {
      flush_long();
      return;
    }
    const int64_t r = (int64_t)(cur_row - key_base);
    uint32_t* row_words = dst_base + r * dst_row_words;
#pragma unroll
    for (int p = 0; p < PPL; ++p) {
      if (!piece_ok[p]) continue;
      double d[EPP];
#pragma unroll
      for (int i = 0; i < EPP; ++i) d[i] = fix_value(acc[p * EPP + i]);
      if constexpr (kSq) {
        uint32_t* sq_words = sq_base + r * dst_row_words;
        uint32_t old2[WPP];
        load_words<WPP>(sq_words + (int64_t)(p * 64 + lane) * WPP, old2);
        double d2[EPP];
#pragma unroll
        for (int i = 0; i < EPP; ++i) {
          d2[i] = (double)a.c2 * d[i] * d[i];
          d[i] *= (double)a.c1;
        }
        write_piece(row_words, p, old[p], d);
        write_piece(sq_words, p, old2, d2);
      } else {
        write_piece(row_words, p, old[p], d);
      }
    }
  };

  for (int64_t q = begin; q < end; q += 64) {
    Term t;
    t.row = kNoRow; t.center = 0; t.coef = 0.f; t.pos = 0;
    if (q + lane < end) t = sorted[q + lane];
    const int n = (int)min((int64_t)64, end - q);
#pragma unroll 1
    for (int b0 = 0; b0 < n; b0 += UB) {
      uint32_t u[UB][PPL][SW];
#pragma unroll
      for (int b = 0; b < UB; ++b) {
        if (b0 + b < n) {
          const int64_t src = (int64_t)__builtin_amdgcn_readlane(t.center, b0 + b);
          const uint32_t* row_words = src_base + src * src_row_words;
#pragma unroll
          for (int p = 0; p < PPL; ++p) {
            if (piece_ok[p]) {
              load_words<SW>(row_words + (int64_t)(p * 64 + lane) * SW, u[b][p]);
            } else {
#pragma unroll
              for (int w = 0; w < SW; ++w) u[b][p][w] = 0u;
            }
          }
        }
      }
#pragma unroll
      for (int b = 0; b < UB; ++b) {
        if (b0 + b < n) {
          const uint32_t pos = (uint32_t)__builtin_amdgcn_readlane((int)t.pos, b0 + b);
          if ((pos & seg_mask) == 0u) {                  // a segment starts here
            const uint32_t row = (uint32_t)__builtin_amdgcn_readlane((int)t.row, b0 + b);
            if (cur_row != kNoRow) flush(row == cur_row);
            cur_row = row;
            cur_seg = pos >> a.seg_shift;
            seg_first = q + b0 + b;
            cur_terms = 0;
#pragma unroll
            for (int x = 0; x < EPL; ++x) acc[x] = 0;
            if (pos == 0u) {
              const uint32_t* row_words = dst_base + (int64_t)(cur_row - key_base) * dst_row_words;
#pragma unroll
              for (int p = 0; p < PPL; ++p)
                if (piece_ok[p]) load_words<WPP>(row_words + (int64_t)(p * 64 + lane) * WPP, old[p]);
            }
          }
          const double c =
              (double)__uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(t.coef), b0 + b)) *
              kFixScale;
#pragma unroll
          for (int p = 0; p < PPL; ++p)
#pragma unroll
            for (int i = 0; i < EPP; ++i) {
              const float x = kStage ? __uint_as_float(u[b][p][i]) : piece_elem<T, SW>(u[b][p], i);
              fix_add(acc[p * EPP + i], c, x);
            }
          ++cur_terms;
        }
      }
    }
  }
  // last pending segment: the row goes on if the term after the range has the same key
  if (cur_row != kNoRow) flush(end < pos_hi && uniform_u32(sorted[end].row) == cur_row);
  }
}

// element-wise row helpers for the finishing kernel (natural order)
__device__ __forceinline__ float elem_load(const float* row, int e) { return row[e]; }
template <typename T, if_16bit<T> = 0>
__device__ __forceinline__ float elem_load(const T* row, int e) { return T::lo((uint32_t)row[e].bits); }
__device__ __forceinline__ void elem_store(float* row, int e, float v) { row[e] = v; }
template <typename T, if_16bit<T> = 0>
__device__ __forceinline__ void elem_store(T* row, int e, float v) { row[e].bits = (uint16_t)T::round(v); }

// ---- finish: table[row] = round(old + side buffer) for the long rows ------------------------
// Side-buffer slot s belongs to the long row (more than one segment of S = 2^seg_shift terms)
// whose first term lies in [s * S, (s+1) * S): that row then also owns the last position of
// the window.  The last block of the launch adds up the per-block
// loss partials instead (in a fixed order, so the loss is reproducible); a bad id
// or an out-of-range product seen by an earlier kernel turns it into NaN.
// which: 0 = long rows of both tables and the loss; 1 = context-table keys only, no loss;
// 2 = input-table keys and the loss.  With one table on both sides a row can be long under
// both of its keys, and its two read-modify-writes must not overlap: the context-table keys
// are then finished before the input-table keys are summed.
template <typename T>
__global__ __launch_bounds__(kSgnsThreads) void sgns_finish_kernel(SgnsArgs a, int which) {
  if (blockIdx.x == gridDim.x - 1) {
    if (which == 1) return;
    __shared__ double sum_s[kSgnsThreads];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < a.forward_blocks; i += kSgnsThreads) acc += a.loss_partials[i];
    sum_s[threadIdx.x] = acc;
    __syncthreads();
    for (int w = kSgnsThreads / 2; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) sum_s[threadIdx.x] += sum_s[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0)
      *a.loss_out = (*a.bad_ids != 0u) ? __longlong_as_double(0x7ff8000000000000ll) : sum_s[0];
    return;
  }
  const int l16 = threadIdx.x & (kGroupLanes - 1);
  const int64_t s = ((int64_t)blockIdx.x * kSgnsThreads + threadIdx.x) / kGroupLanes;
  const int64_t last_pos = ((s + 1) << a.seg_shift) - 1;
  const int64_t total = (int64_t)a.cnt[a.cnt_last];
  if (last_pos >= total) return;
  const Term t = a.sorted[last_pos];
  const int64_t first_pos = last_pos - (int64_t)t.pos;
  if ((first_pos >> a.seg_shift) != s) return;
  // long: the row has a term at position S
  const int64_t second = first_pos + ((int64_t)1 << a.seg_shift);
  if (second >= total || a.sorted[second].row != t.row) return;
  const bool input_row = (int64_t)t.row >= a.num_nodes;
  if (which != 0 && input_row != (which == 2)) return;
  const int64_t row = input_row ? (int64_t)t.row - a.num_nodes : (int64_t)t.row;
  const unsigned long long* src = reinterpret_cast<const unsigned long long*>(a.long_acc) + s * (int64_t)a.dim;
  T* dst = static_cast<T*>(input_row ? a.dst_in : a.dst_out) + row * (int64_t)a.dim;
  float* sq = input_row ? a.sq_in : a.sq_out;
  if (sq != nullptr) {
    sq += row * (int64_t)a.dim;
    for (int e = l16; e < a.dim; e += kGroupLanes) {
      const double d = fix_value(src[e]);
      elem_store(dst, e, (float)((double)elem_load(dst, e) + (double)a.c1 * d));
      sq[e] = (float)((double)sq[e] + (double)a.c2 * d * d);
    }
    return;
  }
  for (int e = l16; e < a.dim; e += kGroupLanes)
    elem_store(dst, e, (float)((double)elem_load(dst, e) + fix_value(src[e])));
}

// ---- host side -----------------------------------------------------------------------------
// Work per 16-lane group: large batches fill the chip many times over, so long runs per
// group amortise the row loads of a run of equal centres; small batches are cut finer so
// that every compute unit gets work and the dependent loads of a group stay few.
static int chunk_pairs_for(int64_t num_pairs) {
  return num_pairs >= (1 << 20) ? 16 : (num_pairs >= (1 << 18) ? 8 : 4);
}
static int slice_terms_for(int64_t num_pairs) {
  return num_pairs >= (1 << 20) ? 128 : (num_pairs >= (1 << 18) ? 64 : 32);
}
static int seg_shift_for(int64_t num_pairs) {
  return num_pairs >= (1 << 18) ? kSegShiftLarge : kSegShiftSmall;
}
static int64_t forward_blocks_for(int64_t num_pairs) {
  return ceil_div(ceil_div(num_pairs, chunk_pairs_for(num_pairs)), kGroupsPerBlock);
}

struct SgnsPlan {
  double* loss_partials;
  float* g;
  uint32_t* rank;
  uint32_t* cnt;
  int64_t cnt_last;         // counters are cnt[0 .. cnt_last]
  uint32_t* key_table;      // tables of the batch's keys (null: none)
  int64_t table_places;
  int32_t out_bits, in_bits;
  uint32_t in_base;
  uint32_t* tile_sums;
  uint32_t* bad_ids;
  Term* sorted;
  long long* long_acc;
  int32_t* stage_center;
  uint32_t* stage_rank;
  float* stage_delta;
  int64_t long_slots;
  int32_t seg_shift;
  size_t bytes;
};

// force_compact: always count over the table of the batch's keys, whatever the graph's size,
// so that the workspace depends on (num_pairs, k, dim) only
static SgnsPlan plan_sgns(void* ws, int64_t num_pairs, int64_t num_nodes, int32_t k, int32_t dim,
                          bool force_compact = false) {
  Carver cv(ws);
  SgnsPlan p;
  const size_t b = (size_t)(num_pairs > 0 ? num_pairs : 1);
  const size_t terms = b * (size_t)(k + 1);
  const size_t keys = 2 * (size_t)(num_nodes > 0 ? num_nodes : 1);
  // A counter per key while the keys are few.  For graphs much larger than the batch (the
  // paper's own batches of 512 to 2048 source nodes on graphs of 10^8 and more vertices) the
  // counters go over the places of a table of the keys the batch holds (at most one per term
  // and per pair): everything that is cleared, scanned or hit at random in a call then has
  // the size of the batch, not of the graph.
  // (a table has at least twice as many places as there can be keys of its kind)
  const size_t nodes = keys / 2;
  const bool compact = force_compact || keys > kCompactFactor * (terms + b);
  int in_bits = 8, out_bits = 8;
  while (((size_t)1 << out_bits) < 2 * terms) ++out_bits;
  while (((size_t)1 << in_bits) < 2 * b) ++in_bits;
  p.out_bits = compact ? out_bits : 0;
  p.in_bits = (compact || ((size_t)1 << in_bits) < nodes) ? in_bits : 0;
  const size_t out_slots = p.out_bits ? (size_t)1 << p.out_bits : nodes;
  const size_t in_slots = p.in_bits ? (size_t)1 << p.in_bits : nodes;
  p.in_base = (uint32_t)out_slots;
  p.table_places = (int64_t)((p.out_bits ? (size_t)1 << p.out_bits : 0) + (p.in_bits ? (size_t)1 << p.in_bits : 0));
  p.cnt_last = (int64_t)(out_slots + in_slots);
  p.seg_shift = seg_shift_for((int64_t)b);
  p.long_slots = (int64_t)((terms + b) >> p.seg_shift) + 1;
  p.loss_partials = cv.take<double>((size_t)forward_blocks_for((int64_t)b));
  p.g = cv.take<float>(terms);
  p.rank = cv.take<uint32_t>(terms);
  p.cnt = cv.take<uint32_t>((size_t)p.cnt_last + 1 + 3);                   // cleared 16 bytes at a time
  p.key_table = p.table_places > 0 ? cv.take<uint32_t>((size_t)p.table_places) : nullptr;
  p.tile_sums = cv.take<uint32_t>((size_t)ceil_div(p.cnt_last + 1, kScanTile));
  p.bad_ids = cv.take<uint32_t>(1);
  p.sorted = cv.take<Term>(terms + b);
  p.long_acc = cv.take<long long>((size_t)p.long_slots * (size_t)dim);
  p.stage_center = cv.take<int32_t>(b);
  p.stage_rank = cv.take<uint32_t>(b);
  p.stage_delta = cv.take<float>(b * (size_t)dim);
  p.bytes = cv.used;
  return p;
}

// the two update passes (context-table keys, then input-table keys) in the piece layout that
// fits the row: 64 lanes x WPP words x PPL pieces cover the row, UB source rows in flight
template <typename T, int WPP, int PPL, int UB>
static int32_t launch_updates(const SgnsArgs& a, hipStream_t stream) {
  constexpr int kWaves = kSgnsThreads / 64;
  // context-table keys: exactly num_terms positions; input-table keys: at most one per pair
  const unsigned out_blocks = (unsigned)ceil_div(ceil_div(a.num_terms, a.slice_terms), kWaves);
  const unsigned in_blocks = (unsigned)min((int64_t)kStageMaxBlocks, ceil_div(ceil_div(a.num_pairs, kStageSlice), kWaves));
  const size_t lds = 0;
  const unsigned finish_blocks = (unsigned)ceil_div(a.long_slots, kGroupsPerBlock) + 1;
  const bool one_table = a.snap != nullptr;
  if constexpr (std::is_same<T, float>::value) {
    if (a.sq_out != nullptr) {
      sgns_update_kernel<T, WPP, PPL, UB, true, false><<<out_blocks, kSgnsThreads, lds, stream>>>(a);
      sgns_update_kernel<T, WPP, PPL, UB, true, true><<<in_blocks, kSgnsThreads, lds, stream>>>(a);
      GS_LAUNCH_CHECK();
      return GS_OK;
    }
  }
  sgns_update_kernel<T, WPP, PPL, UB, false, false><<<out_blocks, kSgnsThreads, lds, stream>>>(a);
  if (one_table) sgns_finish_kernel<T><<<finish_blocks, kSgnsThreads, 0, stream>>>(a, 1);
  sgns_update_kernel<T, WPP, PPL, UB, false, true><<<in_blocks, kSgnsThreads, lds, stream>>>(a);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

template <typename T, int VPL, int RB>
static int32_t launch_sgns(const SgnsArgs& a, hipStream_t stream) {
  const int64_t keys1 = a.cnt_last + 1;
  const int64_t tiles = ceil_div(keys1, kScanTile);
  const int64_t keys4 = ceil_div(keys1, 4);
  const int64_t table4 = a.table_places / 4;   // (tables have at least 256 places each)
  sgns_clear_kernel<<<(unsigned)ceil_div(max(keys4, table4), 256), 256, 0, stream>>>(
      (uint4*)a.cnt, keys4, (uint4*)a.key_table, table4, a.bad_ids);
  GS_LAUNCH_CHECK();
  const size_t idx_lds = (size_t)kGroupsPerBlock * a.chunk_pairs * (a.k + 2) * sizeof(int32_t);
  sgns_forward_kernel<T, VPL, RB><<<(unsigned)(a.forward_blocks_per_xcd * 8), kSgnsThreads, idx_lds,
                                   stream>>>(a);
  GS_LAUNCH_CHECK();
  if (keys1 <= kScanSmallMax) {
    scan_small_kernel<<<1, 1024, 0, stream>>>(a.cnt, keys1);
    GS_LAUNCH_CHECK();
  } else {
    scan_reduce_kernel<<<(unsigned)tiles, kScanThreads, 0, stream>>>(a.cnt, keys1, a.tile_sums);
    GS_LAUNCH_CHECK();
    const int raw_sums = tiles <= kFewTiles ? 1 : 0;
    if (!raw_sums) {
      scan_tiles_kernel<<<1, 1024, 0, stream>>>(a.tile_sums, tiles);
      GS_LAUNCH_CHECK();
    }
    scan_apply_kernel<<<(unsigned)tiles, kScanThreads, 0, stream>>>(a.cnt, keys1, a.tile_sums, raw_sums);
    GS_LAUNCH_CHECK();
  }
  sgns_place_kernel<<<(unsigned)ceil_div(a.num_terms + a.num_pairs, 256), 256, 0, stream>>>(a);
  GS_LAUNCH_CHECK();
  const int row_bytes = a.dim * (int)sizeof(T);
  int32_t rc;
  if (row_bytes <= 256) rc = launch_updates<T, 1, 1, 16>(a, stream);
  else if (row_bytes <= 512) rc = launch_updates<T, 2, 1, 16>(a, stream);
  else if (row_bytes <= 1024) rc = launch_updates<T, 4, 1, 8>(a, stream);
  else if (row_bytes <= 2048) rc = launch_updates<T, 4, 2, 4>(a, stream);
  else rc = launch_updates<T, 4, 4, 2>(a, stream);
  if (rc != GS_OK) return rc;
  // long rows (of both tables, unless the context-table ones are done); one more block sums the loss
  const unsigned finish_blocks = (unsigned)ceil_div(a.long_slots, kGroupsPerBlock) + 1;
  sgns_finish_kernel<T><<<finish_blocks, kSgnsThreads, 0, stream>>>(a, a.snap != nullptr ? 2 : 0);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

__global__ void zero_double_kernel(double* p) { *p = 0.0; }

// ---- dense passes of the momentum step (16 bytes per lane, grid-stride) ----------------
// momentum <- mu * momentum over a whole table ("mult" of GraphScale Sec. 3.2)
__global__ __launch_bounds__(256) void table_scale_kernel(float4* __restrict__ m, int64_t n4, float mu) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    float4 x = m[i];
    x.x *= mu; x.y *= mu; x.z *= mu; x.w *= mu;
    m[i] = x;
  }
}
template <typename T>
__global__ __launch_bounds__(256) void table_scale16_kernel(uint4* __restrict__ m, int64_t n8, float mu) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8;
       i += (int64_t)gridDim.x * blockDim.x) {
    uint4 x = m[i];
    x.x = pack16<T>(T::lo(x.x) * mu, T::hi(x.x) * mu);
    x.y = pack16<T>(T::lo(x.y) * mu, T::hi(x.y) * mu);
    x.z = pack16<T>(T::lo(x.z) * mu, T::hi(x.z) * mu);
    x.w = pack16<T>(T::lo(x.w) * mu, T::hi(x.w) * mu);
    m[i] = x;
  }
}
// model <- model - lr * momentum over a whole table ("mult_add")
__global__ __launch_bounds__(256) void table_axpy_kernel(float4* __restrict__ w,
                                                         const float4* __restrict__ m, int64_t n4,
                                                         float lr) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    float4 x = w[i];
    const float4 y = m[i];
    x.x -= lr * y.x; x.y -= lr * y.y; x.z -= lr * y.z; x.w -= lr * y.w;
    w[i] = x;
  }
}
template <typename T>
__global__ __launch_bounds__(256) void table_axpy16_kernel(uint4* __restrict__ w,
                                                           const uint4* __restrict__ m, int64_t n8,
                                                           float lr) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8;
       i += (int64_t)gridDim.x * blockDim.x) {
    uint4 x = w[i];
    const uint4 y = m[i];
    x.x = pack16<T>(T::lo(x.x) - lr * T::lo(y.x), T::hi(x.x) - lr * T::hi(y.x));
    x.y = pack16<T>(T::lo(x.y) - lr * T::lo(y.y), T::hi(x.y) - lr * T::hi(y.y));
    x.z = pack16<T>(T::lo(x.z) - lr * T::lo(y.z), T::hi(x.z) - lr * T::hi(y.z));
    x.w = pack16<T>(T::lo(x.w) - lr * T::lo(y.w), T::hi(x.w) - lr * T::hi(y.w));
    w[i] = x;
  }
}

// Adam's dense passes over a whole fp32 table: decay of both moments, then the model update
__global__ __launch_bounds__(256) void adam_decay_kernel(float4* __restrict__ m, float4* __restrict__ v,
                                                         int64_t n4, float beta1, float beta2) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    float4 x = m[i], y = v[i];
    x.x *= beta1; x.y *= beta1; x.z *= beta1; x.w *= beta1;
    y.x *= beta2; y.y *= beta2; y.z *= beta2; y.w *= beta2;
    m[i] = x;
    v[i] = y;
  }
}
__device__ __forceinline__ float adam_move(float m, float v, float step, float root_c2, float eps) {
  return step * m / (sqrtf(v) / root_c2 + eps);
}
__global__ __launch_bounds__(256) void adam_apply_kernel(float4* __restrict__ w,
                                                         const float4* __restrict__ m,
                                                         const float4* __restrict__ v, int64_t n4,
                                                         float step, float root_c2, float eps) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    float4 x = w[i];
    const float4 a = m[i], b = v[i];
    x.x -= adam_move(a.x, b.x, step, root_c2, eps);
    x.y -= adam_move(a.y, b.y, step, root_c2, eps);
    x.z -= adam_move(a.z, b.z, step, root_c2, eps);
    x.w -= adam_move(a.w, b.w, step, root_c2, eps);
    w[i] = x;
  }
}

static int32_t check_sgns_args(const void* w_in, const void* w_out, int64_t num_nodes, int32_t dim,
                               int32_t dtype, const int32_t* centers, const int32_t* contexts,
                               const int32_t* negs, int64_t num_pairs, int32_t k,
                               const double* loss_sum_out, const void* ws, bool one_table = false) {
  if (!w_in || !w_out || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX) return GS_EINVAL;
  if (dtype != GS_F32 && dtype != GS_BF16 && dtype != GS_F16) return GS_EINVAL;
  const int granule = (dtype == GS_F32) ? 4 : 8;   // elements per 16-byte piece
  if (dim < granule || dim > 1024 || (dim % granule) != 0) return GS_EINVAL;
  if (num_pairs < 0 || k < 0 || k > 60 || !loss_sum_out) return GS_EINVAL;
  if (num_pairs > 0 && (!centers || !contexts || (k > 0 && !negs))) return GS_EINVAL;
  if (num_pairs * (int64_t)(k + 1) > (int64_t)0x7fffffff) return GS_EOVERFLOW;
  if (!aligned(w_in, 16) || !aligned(w_out, 16)) return GS_EINVAL;
  if (w_in == w_out && !one_table) return GS_EINVAL;   // needs the one-table entry point
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  return GS_OK;
}

// What the variants of the step add to the plain one.
struct SgnsExtras {
  float* sq_in = nullptr;          // Adam: second-moment tables and the two put coefficients
  float* sq_out = nullptr;
  float c1 = 1.f, c2 = 0.f;
  const gs_alias* noise = nullptr; // negatives drawn inside the step (negs_draw != null)
  uint64_t neg_seed = 0, neg_pair_base = 0;
  int32_t* negs_draw = nullptr;
  void* snap = nullptr;            // one table on both sides: copies of the input rows, pair slots
  int32_t* pair_slot = nullptr;
  const int32_t* walks = nullptr;  // pairs made inside the step
  const int64_t* pair_offsets = nullptr;
  int64_t num_walks = 0, first_pair = 0;
  int32_t walk_len = 0, window = 0;
  int32_t* gen_centers = nullptr;
  int32_t* gen_contexts = nullptr;
};

// Logits from (w_in, w_out); every touched row r of the destination tables becomes
// round(dst[r] - lr * gradient_r).  Plain SGD: destination = the tables themselves.
static int32_t run_sgns(void* w_in, void* w_out, void* dst_in, void* dst_out, int64_t num_nodes,
                        int32_t dim, int32_t dtype, const int32_t* centers, const int32_t* contexts,
                        const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                        double* loss_sum_out, const SgnsPlan& p, hipStream_t stream,
                        const SgnsExtras& x = SgnsExtras()) {
  SgnsArgs a;
  a.sq_in = x.sq_in;
  a.sq_out = x.sq_out;
  a.c1 = x.c1;
  a.c2 = x.c2;
  a.draw_negs = x.negs_draw != nullptr ? 1 : 0;
  const bool weighted = x.noise != nullptr && x.noise->prob != nullptr;
  a.noise_prob = weighted ? x.noise->prob : nullptr;
  a.noise_alias = weighted ? x.noise->alias : nullptr;
  a.noise_packed = weighted ? reinterpret_cast<const uint2*>(x.noise->packed) : nullptr;
  a.neg_seed = x.neg_seed;
  a.neg_pair_base = x.neg_pair_base;
  a.negs_draw = x.negs_draw;
  if (a.draw_negs) negs = x.negs_draw;
  a.snap = x.snap;
  a.pair_slot = x.pair_slot;
  a.walks = x.walks;
  a.pair_offsets = x.pair_offsets;
  a.num_walks = x.num_walks;
  a.first_pair = x.first_pair;
  a.walk_len = x.walk_len;
  a.window = x.window;
  a.gen_centers = x.gen_centers;
  a.gen_contexts = x.gen_contexts;
  if (a.walks != nullptr) {
    centers = x.gen_centers;
    contexts = x.gen_contexts;
  }
  a.w_in = w_in;
  a.w_out = w_out;
  a.dst_in = dst_in;
  a.dst_out = dst_out;
  a.centers = centers;
  a.contexts = contexts;
  a.negs = negs;
  a.num_pairs = num_pairs;
  a.num_nodes = num_nodes;
  a.num_terms = num_pairs * (int64_t)(k + 1);
  a.long_slots = p.long_slots;
  a.seg_shift = p.seg_shift;
  a.k = k;
  a.dim = dim;
  a.lr = lr;
  a.g = p.g;
  a.rank = p.rank;
  a.cnt = p.cnt;
  a.cnt_last = p.cnt_last;
  a.key_table = p.key_table;
  a.table_places = p.table_places;
  a.out_bits = p.out_bits;
  a.in_bits = p.in_bits;
  a.in_base = p.in_base;
  a.tile_sums = p.tile_sums;
  a.bad_ids = p.bad_ids;
  a.sorted = p.sorted;
  a.long_acc = p.long_acc;
  a.stage_center = p.stage_center;
  a.stage_rank = p.stage_rank;
  a.stage_delta = p.stage_delta;
  a.chunk_pairs = chunk_pairs_for(num_pairs);
  a.slice_terms = slice_terms_for(num_pairs);
  a.loss_partials = p.loss_partials;
  a.forward_blocks = forward_blocks_for(num_pairs);
  a.forward_blocks_per_xcd = ceil_div(a.forward_blocks, 8);
  a.loss_out = loss_sum_out;
  // float4 registers per lane for one row: 16 lanes x 4 floats = 64 elements each
  const int vpl = (dim + 63) / 64;
  if (dtype == GS_F32) {
    if (vpl <= 1) return launch_sgns<float, 1, 6>(a, stream);
    if (vpl <= 2) return launch_sgns<float, 2, 6>(a, stream);
    if (vpl <= 4) return launch_sgns<float, 4, 3>(a, stream);
    if (vpl <= 8) return launch_sgns<float, 8, 2>(a, stream);
    return launch_sgns<float, 16, 1>(a, stream);
  }
  // 16-bit rows: a 16-byte piece is 8 elements = two float4, so the register count is even
  if (dtype == GS_BF16) {
    if (vpl <= 2) return launch_sgns<bf16_t, 2, 6>(a, stream);
    if (vpl <= 4) return launch_sgns<bf16_t, 4, 6>(a, stream);
    if (vpl <= 8) return launch_sgns<bf16_t, 8, 4>(a, stream);
    return launch_sgns<bf16_t, 16, 2>(a, stream);
  }
  if (vpl <= 2) return launch_sgns<f16_t, 2, 6>(a, stream);
  if (vpl <= 4) return launch_sgns<f16_t, 4, 6>(a, stream);
  if (vpl <= 8) return launch_sgns<f16_t, 8, 4>(a, stream);
  return launch_sgns<f16_t, 16, 2>(a, stream);
}

}  // namespace gs

using namespace gs;

extern "C" size_t gs_sgns_step_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                               int32_t dim, int32_t dtype) {
  (void)dtype;
  if (num_pairs < 0 || num_nodes < 0 || k < 0 || dim < 1) return 0;
  return plan_sgns(nullptr, num_pairs, num_nodes, k, dim).bytes;
}

extern "C" int32_t gs_sgns_step(void* w_in, void* w_out, int64_t num_nodes, int32_t dim,
                                int32_t dtype, const int32_t* centers, const int32_t* contexts,
                                const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                double* loss_sum_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs,
                                      num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  return run_sgns(w_in, w_out, w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs, num_pairs,
                  k, lr, loss_sum_out, p, stream);
}

// ---- the step for callers that cannot allocate ------------------------------------------
// Scratch memory of gs_sgns_step_static: one array per GPU, part of the loaded code object,
// held until the process ends.  Host code never uses the array's name as an address: the
// device address is asked for once per device (hipGetSymbolAddress, with that device
// current) and kept.
constexpr int64_t kStaticMaxPairs = 4096;
constexpr int64_t kStaticMaxTerms = 65536;
constexpr int32_t kStaticMaxDim = 256;
constexpr size_t kStaticScratchBytes = (size_t)12 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

constexpr int kStaticMaxDevices = 64;
static void* g_scratch_ptr[kStaticMaxDevices];   // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

static int32_t static_scratch(void** out) {
  int dev = -1;
  GS_HIP_TRY(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) return GS_EINVAL;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    GS_HIP_TRY(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return GS_EHIP;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return GS_OK;
}

extern "C" int32_t gs_sgns_step_static(void* w_in, void* w_out, int64_t num_nodes, int32_t dim,
                                       int32_t dtype, const int32_t* centers, const int32_t* contexts,
                                       const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                       double* loss_sum_out, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (num_pairs > kStaticMaxPairs || dim > kStaticMaxDim) return GS_EWORKSPACE;
  if (num_pairs > 0 && k >= 0 && num_pairs * (int64_t)(k + 1) > kStaticMaxTerms) return GS_EWORKSPACE;
  void* ws = nullptr;
  const int32_t got = static_scratch(&ws);
  if (got != GS_OK) return got;
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs,
                                      num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim, true);
  if (p.bytes > kStaticScratchBytes) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  return run_sgns(w_in, w_out, w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs, num_pairs,
                  k, lr, loss_sum_out, p, stream);
}

// workspace of the fused call: the step's own, then the drawn negatives
static size_t fused_negs_bytes(int64_t num_pairs, int32_t k) {
  return align_up((size_t)(num_pairs > 0 ? num_pairs : 1) * (size_t)(k > 0 ? k : 1) * sizeof(int32_t));
}

extern "C" size_t gs_sgns_step_fused_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                                     int32_t dim, int32_t dtype) {
  (void)dtype;
  if (num_pairs < 0 || num_nodes < 0 || k < 0 || dim < 1) return 0;
  return plan_sgns(nullptr, num_pairs, num_nodes, k, dim).bytes + fused_negs_bytes(num_pairs, k);
}

extern "C" int32_t gs_sgns_step_fused(void* w_in, void* w_out, int64_t num_nodes, int32_t dim,
                                      int32_t dtype, const int32_t* centers, const int32_t* contexts,
                                      int64_t num_pairs, const gs_alias* noise,
                                      uint64_t pair_index_base, uint64_t neg_seed, int32_t k, float lr,
                                      double* loss_sum_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  // the negatives live in the workspace: hand the checker a non-null stand-in
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, dtype, centers, contexts,
                                      static_cast<const int32_t*>(ws), num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  if (noise != nullptr && noise->prob != nullptr && !noise->alias) return GS_EINVAL;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  if (ws_bytes < p.bytes + fused_negs_bytes(num_pairs, k)) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  int32_t* negs_ws = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.bytes);
  SgnsExtras x;
  x.noise = noise;
  x.neg_seed = neg_seed;
  x.neg_pair_base = pair_index_base;
  x.negs_draw = negs_ws;
  return run_sgns(w_in, w_out, w_in, w_out, num_nodes, dim, dtype, centers, contexts, nullptr,
                  num_pairs, k, lr, loss_sum_out, p, stream, x);
}

// workspace of the call that makes its pairs: the step's own, the drawn negatives, the derived ids
static size_t walk_ids_bytes(int64_t num_pairs) {
  return align_up((size_t)(num_pairs > 0 ? num_pairs : 1) * sizeof(int32_t));
}

extern "C" size_t gs_sgns_step_from_walks_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                                          int32_t dim, int32_t dtype) {
  (void)dtype;
  if (num_pairs < 0 || num_nodes < 0 || k < 0 || dim < 1) return 0;
  return plan_sgns(nullptr, num_pairs, num_nodes, k, dim).bytes + fused_negs_bytes(num_pairs, k) +
         2 * walk_ids_bytes(num_pairs);
}

extern "C" int32_t gs_sgns_step_from_walks(void* w_in, void* w_out, int64_t num_nodes, int32_t dim,
                                           int32_t dtype, const int32_t* walks, int64_t num_walks,
                                           int32_t walk_len, int32_t window, const int64_t* pair_offsets,
                                           int64_t first_pair, int64_t num_pairs, const gs_alias* noise,
                                           uint64_t pair_index_base, uint64_t neg_seed, int32_t k,
                                           float lr, double* loss_sum_out, void* ws, size_t ws_bytes,
                                           void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!walks || !pair_offsets || num_walks < 1 || walk_len < 1 || walk_len > 4096 || window < 1 ||
      first_pair < 0)
    return GS_EINVAL;
  // the ids live in the workspace: hand the checker non-null stand-ins
  const int32_t* stand_in = static_cast<const int32_t*>(ws);
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, dtype, stand_in, stand_in, stand_in,
                                      num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  if (noise != nullptr && noise->prob != nullptr && !noise->alias) return GS_EINVAL;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  const size_t negs_bytes = fused_negs_bytes(num_pairs, k), ids_bytes = walk_ids_bytes(num_pairs);
  if (ws_bytes < p.bytes + negs_bytes + 2 * ids_bytes) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  char* extra = static_cast<char*>(ws) + p.bytes;
  SgnsExtras x;
  x.noise = noise;
  x.neg_seed = neg_seed;
  x.neg_pair_base = pair_index_base;
  x.negs_draw = reinterpret_cast<int32_t*>(extra);
  x.gen_centers = reinterpret_cast<int32_t*>(extra + negs_bytes);
  x.gen_contexts = reinterpret_cast<int32_t*>(extra + negs_bytes + ids_bytes);
  x.walks = walks;
  x.pair_offsets = pair_offsets;
  x.num_walks = num_walks;
  x.first_pair = first_pair;
  x.walk_len = walk_len;
  x.window = window;
  return run_sgns(w_in, w_out, w_in, w_out, num_nodes, dim, dtype, nullptr, nullptr, nullptr, num_pairs,
                  k, lr, loss_sum_out, p, stream, x);
}

// workspace of the one-table step: the step's own, the copies of the input rows, the pair slots
static size_t line1_snap_bytes(int64_t num_pairs, int32_t dim, int32_t dtype) {
  return align_up((size_t)(num_pairs > 0 ? num_pairs : 1) * (size_t)dim * (dtype == GS_F32 ? 4 : 2));
}
static size_t line1_slot_bytes(int64_t num_pairs) {
  return align_up((size_t)(num_pairs > 0 ? num_pairs : 1) * sizeof(int32_t));
}

extern "C" size_t gs_line1_step_workspace_bytes(int64_t num_pairs, int64_t num_nodes, int32_t k,
                                                int32_t dim, int32_t dtype) {
  if (num_pairs < 0 || num_nodes < 0 || k < 0 || dim < 1) return 0;
  return plan_sgns(nullptr, num_pairs, num_nodes, k, dim).bytes +
         line1_snap_bytes(num_pairs, dim, dtype) + line1_slot_bytes(num_pairs);
}

extern "C" int32_t gs_line1_step(void* w, int64_t num_nodes, int32_t dim, int32_t dtype,
                                 const int32_t* sources, const int32_t* targets, const int32_t* negs,
                                 int64_t num_pairs, int32_t k, float lr, double* loss_sum_out,
                                 void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t bad = check_sgns_args(w, w, num_nodes, dim, dtype, sources, targets, negs, num_pairs,
                                      k, loss_sum_out, ws, true);
  if (bad != GS_OK) return bad;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  const size_t snap_bytes = line1_snap_bytes(num_pairs, dim, dtype);
  if (ws_bytes < p.bytes + snap_bytes + line1_slot_bytes(num_pairs)) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  SgnsExtras x;
  x.snap = static_cast<char*>(ws) + p.bytes;
  x.pair_slot = reinterpret_cast<int32_t*>(static_cast<char*>(ws) + p.bytes + snap_bytes);
  return run_sgns(w, w, w, w, num_nodes, dim, dtype, sources, targets, negs, num_pairs, k, lr,
                  loss_sum_out, p, stream, x);
}

extern "C" int32_t gs_sgns_momentum_step(void* w_in, void* w_out, void* m_in, void* m_out,
                                         int64_t num_nodes, int32_t dim, int32_t dtype,
                                         const int32_t* centers, const int32_t* contexts,
                                         const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                         float mu, double* loss_sum_out, void* ws, size_t ws_bytes,
                                         void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, dtype, centers, contexts, negs,
                                      num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  if (!m_in || !m_out || !aligned(m_in, 16) || !aligned(m_out, 16)) return GS_EINVAL;
  if (m_in == w_in || m_in == w_out || m_out == w_in || m_out == w_out || m_in == m_out)
    return GS_EINVAL;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  const int per16 = (dtype == GS_F32) ? 4 : 8;
  const int64_t pieces = num_nodes * (int64_t)dim / per16;
  const unsigned blocks = (unsigned)min((int64_t)(256 * 64), ceil_div(pieces, 256));
  // mult: momentum <- mu * momentum, every row
  if (dtype == GS_F32) {
    table_scale_kernel<<<blocks, 256, 0, stream>>>((float4*)m_in, pieces, mu);
    table_scale_kernel<<<blocks, 256, 0, stream>>>((float4*)m_out, pieces, mu);
  } else if (dtype == GS_BF16) {
    table_scale16_kernel<bf16_t><<<blocks, 256, 0, stream>>>((uint4*)m_in, pieces, mu);
    table_scale16_kernel<bf16_t><<<blocks, 256, 0, stream>>>((uint4*)m_out, pieces, mu);
  } else {
    table_scale16_kernel<f16_t><<<blocks, 256, 0, stream>>>((uint4*)m_in, pieces, mu);
    table_scale16_kernel<f16_t><<<blocks, 256, 0, stream>>>((uint4*)m_out, pieces, mu);
  }
  GS_LAUNCH_CHECK();
  // put: momentum[rows of the batch] += gradient (the update machinery with step -1)
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
  } else {
    const int32_t rc = run_sgns(w_in, w_out, m_in, m_out, num_nodes, dim, dtype, centers, contexts,
                                negs, num_pairs, k, -1.0f, loss_sum_out, p, stream);
    if (rc != GS_OK) return rc;
  }
  // mult_add: model <- model - lr * momentum, every row
  if (dtype == GS_F32) {
    table_axpy_kernel<<<blocks, 256, 0, stream>>>((float4*)w_in, (const float4*)m_in, pieces, lr);
    table_axpy_kernel<<<blocks, 256, 0, stream>>>((float4*)w_out, (const float4*)m_out, pieces, lr);
  } else if (dtype == GS_BF16) {
    table_axpy16_kernel<bf16_t><<<blocks, 256, 0, stream>>>((uint4*)w_in, (const uint4*)m_in, pieces, lr);
    table_axpy16_kernel<bf16_t><<<blocks, 256, 0, stream>>>((uint4*)w_out, (const uint4*)m_out, pieces, lr);
  } else {
    table_axpy16_kernel<f16_t><<<blocks, 256, 0, stream>>>((uint4*)w_in, (const uint4*)m_in, pieces, lr);
    table_axpy16_kernel<f16_t><<<blocks, 256, 0, stream>>>((uint4*)w_out, (const uint4*)m_out, pieces, lr);
  }
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" int32_t gs_sgns_adam_step(float* w_in, float* w_out, float* m_in, float* m_out, float* v_in,
                                     float* v_out, int64_t num_nodes, int32_t dim,
                                     const int32_t* centers, const int32_t* contexts,
                                     const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                     float beta1, float beta2, float eps, int64_t t,
                                     double* loss_sum_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t bad = check_sgns_args(w_in, w_out, num_nodes, dim, GS_F32, centers, contexts, negs,
                                      num_pairs, k, loss_sum_out, ws);
  if (bad != GS_OK) return bad;
  float* tables[6] = {w_in, w_out, m_in, m_out, v_in, v_out};
  for (int i = 0; i < 6; ++i) {
    if (!tables[i] || !aligned(tables[i], 16)) return GS_EINVAL;
    for (int j = 0; j < i; ++j)
      if (tables[i] == tables[j]) return GS_EINVAL;
  }
  if (t < 1 || !(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
    return GS_EINVAL;
  SgnsPlan p = plan_sgns(ws, num_pairs, num_nodes, k, dim);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  const int64_t pieces = num_nodes * (int64_t)dim / 4;
  const unsigned blocks = (unsigned)min((int64_t)(256 * 64), ceil_div(pieces, 256));
  // mult: both moments decay, every row
  adam_decay_kernel<<<blocks, 256, 0, stream>>>((float4*)m_in, (float4*)v_in, pieces, beta1, beta2);
  adam_decay_kernel<<<blocks, 256, 0, stream>>>((float4*)m_out, (float4*)v_out, pieces, beta1, beta2);
  GS_LAUNCH_CHECK();
  // put: m[r] += (1 - beta1) g[r], v[r] += (1 - beta2) g[r]^2 for the rows of the batch
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
  } else {
    SgnsExtras x;
    x.sq_in = v_in;
    x.sq_out = v_out;
    x.c1 = 1.0f - beta1;
    x.c2 = 1.0f - beta2;
    const int32_t rc = run_sgns(w_in, w_out, m_in, m_out, num_nodes, dim, GS_F32, centers, contexts,
                                negs, num_pairs, k, -1.0f, loss_sum_out, p, stream, x);
    if (rc != GS_OK) return rc;
  }
  // apply: w -= (lr / (1 - beta1^t)) * m / (sqrt(v) / sqrt(1 - beta2^t) + eps), every row
  const float step = (float)((double)lr / (1.0 - pow((double)beta1, (double)t)));
  const float root_c2 = (float)sqrt(1.0 - pow((double)beta2, (double)t));
  adam_apply_kernel<<<blocks, 256, 0, stream>>>((float4*)w_in, (const float4*)m_in,
                                                (const float4*)v_in, pieces, step, root_c2, eps);
  adam_apply_kernel<<<blocks, 256, 0, stream>>>((float4*)w_out, (const float4*)m_out,
                                                (const float4*)v_out, pieces, step, root_c2, eps);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
