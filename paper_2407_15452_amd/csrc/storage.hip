// Storage operations on a batch of vertex ids (GraphScale Sec. 3.1 / 3.2): merge
// equal ids into one request (gs_unique_ids), fetch one n x d block of rows
// (gs_get_rows), add one block of gradient rows to the table (gs_put_rows).
// And the two dense operations of the model update of Sec. 3.2: a table times a
// factor (gs_table_mult), one table plus a factor times another (gs_table_mult_add).
#include "common.h"

namespace gs {

namespace {

constexpr int kRowLanes = 16;                       // lanes per row, 16 bytes each per access
constexpr int kRowThreads = 256;
constexpr int kRowsPerBlock = kRowThreads / kRowLanes;

// id -> sort key; ids that are not rows get the key num_nodes and sort last
__global__ void unique_keys_kernel(const int32_t* __restrict__ ids, int64_t n, int64_t num_nodes,
                                   uint64_t* __restrict__ keys, uint32_t* __restrict__ index) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t v = ids[i];
  keys[i] = (v >= 0 && (int64_t)v < num_nodes) ? (uint64_t)v : (uint64_t)num_nodes;
  index[i] = (uint32_t)i;
}

// head[j] = 1 where a new valid id starts in the sorted keys
__global__ void unique_heads_kernel(const uint64_t* __restrict__ keys, int64_t n, int64_t num_nodes,
                                    int64_t* __restrict__ head) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const uint64_t k = keys[j];
  head[j] = (k < (uint64_t)num_nodes && (j == 0 || keys[j - 1] != k)) ? 1 : 0;
}

// before[j] = number of heads before j (exclusive scan of head)
__global__ void unique_emit_kernel(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ index,
                                   const int64_t* __restrict__ before, int64_t n, int64_t num_nodes,
                                   int32_t* __restrict__ unique_out, int32_t* __restrict__ inverse_out) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const uint64_t k = keys[j];
  const bool valid = k < (uint64_t)num_nodes;
  const bool is_head = valid && (j == 0 || keys[j - 1] != k);
  const int64_t b = before[j];
  if (is_head) unique_out[b] = (int32_t)k;
  if (inverse_out) inverse_out[index[j]] = valid ? (int32_t)(is_head ? b : b - 1) : -1;
}

// ---- merged ids through a bitmap of the node ids (when the batch is not small next to the
// graph): mark, count the bits of every word, scan, then read the ids off in ascending order
__global__ void bitmap_mark_kernel(const int32_t* __restrict__ ids, int64_t n, int64_t num_nodes,
                                   uint32_t* __restrict__ bitmap) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t v = ids[i];
  if (v < 0 || (int64_t)v >= num_nodes) return;
  const uint32_t bit = 1u << (v & 31);
  // bits are only ever set: a word read as already holding the bit needs no atomic (a stale
  // read merely costs a redundant one)
  if ((bitmap[v >> 5] & bit) == 0u) atomicOr(bitmap + (v >> 5), bit);
}

__global__ void bitmap_count_kernel(const uint32_t* __restrict__ bitmap, int64_t words,
                                    int64_t* __restrict__ counts) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w < words) counts[w] = (int64_t)__popc(bitmap[w]);
}

// before[w] = number of set bits in the words before w
__global__ void bitmap_emit_kernel(const uint32_t* __restrict__ bitmap, const int64_t* __restrict__ before,
                                   int64_t words, int32_t* __restrict__ unique_out) {
  const int64_t w = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (w >= words) return;
  uint32_t bits = bitmap[w];
  int64_t at = before[w];
  while (bits != 0u) {
    const int b = __ffs((int)bits) - 1;
    unique_out[at++] = (int32_t)(w * 32 + b);
    bits &= bits - 1u;
  }
}

__global__ void bitmap_inverse_kernel(const int32_t* __restrict__ ids, int64_t n, int64_t num_nodes,
                                      const uint32_t* __restrict__ bitmap,
                                      const int64_t* __restrict__ before,
                                      int32_t* __restrict__ inverse_out) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  const int32_t v = ids[i];
  if (v < 0 || (int64_t)v >= num_nodes) { inverse_out[i] = -1; return; }
  const uint32_t below = bitmap[v >> 5] & ((1u << (v & 31)) - 1u);
  inverse_out[i] = (int32_t)(before[v >> 5] + (int64_t)__popc(below));
}

__global__ void fill_words_kernel(uint32_t* __restrict__ p, int64_t n, uint32_t value) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = value;
}

__device__ __forceinline__ int64_t live_count(int64_t n, const int64_t* count_dev) {
  if (count_dev == nullptr) return n;
  const int64_t c = *count_dev;
  return c < 0 ? 0 : (c < n ? c : n);
}

// round(old + scale * r): exact product and one rounding of the sum in fp64,
// then to fp32 (and from there to the table's 16-bit format)
__device__ __forceinline__ float sum_once(float old, float scale, float r) {
  return (float)((double)old + (double)scale * (double)r);
}

__global__ __launch_bounds__(kRowThreads) void get_rows_f32_kernel(
    const float* __restrict__ table, int64_t num_nodes, int32_t dim, const int32_t* __restrict__ ids,
    int64_t n, const int64_t* __restrict__ count_dev, float* __restrict__ out) {
  const int l16 = threadIdx.x & (kRowLanes - 1);
  const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kRowLanes;
  if (i >= live_count(n, count_dev)) return;
  const int32_t id = ids[i];
  const bool ok = id >= 0 && (int64_t)id < num_nodes;
  const float4* src = reinterpret_cast<const float4*>(table + (int64_t)(ok ? id : 0) * dim);
  float4* dst = reinterpret_cast<float4*>(out + i * (int64_t)dim);
  for (int q = l16; q < (dim >> 2); q += kRowLanes)
    dst[q] = ok ? src[q] : make_float4(0.f, 0.f, 0.f, 0.f);
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void get_rows16_kernel(
    const uint16_t* __restrict__ table, int64_t num_nodes, int32_t dim, const int32_t* __restrict__ ids,
    int64_t n, const int64_t* __restrict__ count_dev, float* __restrict__ out) {
  const int l16 = threadIdx.x & (kRowLanes - 1);
  const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kRowLanes;
  if (i >= live_count(n, count_dev)) return;
  const int32_t id = ids[i];
  const bool ok = id >= 0 && (int64_t)id < num_nodes;
  const uint4* src = reinterpret_cast<const uint4*>(table + (int64_t)(ok ? id : 0) * dim);
  float4* dst = reinterpret_cast<float4*>(out + i * (int64_t)dim);
  for (int c = l16; c < (dim >> 3); c += kRowLanes) {
    const uint4 x = ok ? src[c] : make_uint4(0u, 0u, 0u, 0u);
    dst[2 * c] = make_float4(T::lo(x.x), T::hi(x.x), T::lo(x.y), T::hi(x.y));
    dst[2 * c + 1] = make_float4(T::lo(x.z), T::hi(x.z), T::lo(x.w), T::hi(x.w));
  }
}

__global__ __launch_bounds__(kRowThreads) void put_rows_f32_kernel(
    float* __restrict__ table, int64_t num_nodes, int32_t dim, const int32_t* __restrict__ ids, int64_t n,
    const int64_t* __restrict__ count_dev, const float* __restrict__ rows, float scale) {
  const int l16 = threadIdx.x & (kRowLanes - 1);
  const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kRowLanes;
  if (i >= live_count(n, count_dev)) return;
  const int32_t id = ids[i];
  if (id < 0 || (int64_t)id >= num_nodes) return;
  float4* dst = reinterpret_cast<float4*>(table + (int64_t)id * dim);
  const float4* src = reinterpret_cast<const float4*>(rows + i * (int64_t)dim);
  for (int q = l16; q < (dim >> 2); q += kRowLanes) {
    const float4 o = dst[q], r = src[q];
    dst[q] = make_float4(sum_once(o.x, scale, r.x), sum_once(o.y, scale, r.y),
                         sum_once(o.z, scale, r.z), sum_once(o.w, scale, r.w));
  }
}

template <typename T>
__global__ __launch_bounds__(kRowThreads) void put_rows16_kernel(
    uint16_t* __restrict__ table, int64_t num_nodes, int32_t dim, const int32_t* __restrict__ ids,
    int64_t n, const int64_t* __restrict__ count_dev, const float* __restrict__ rows, float scale) {
  const int l16 = threadIdx.x & (kRowLanes - 1);
  const int64_t i = (int64_t)blockIdx.x * kRowsPerBlock + threadIdx.x / kRowLanes;
  if (i >= live_count(n, count_dev)) return;
  const int32_t id = ids[i];
  if (id < 0 || (int64_t)id >= num_nodes) return;
  uint4* dst = reinterpret_cast<uint4*>(table + (int64_t)id * dim);
  const float4* src = reinterpret_cast<const float4*>(rows + i * (int64_t)dim);
  for (int c = l16; c < (dim >> 3); c += kRowLanes) {
    const uint4 o = dst[c];
    const float4 a = src[2 * c], b = src[2 * c + 1];
    uint4 x;
    x.x = T::round(sum_once(T::lo(o.x), scale, a.x)) | (T::round(sum_once(T::hi(o.x), scale, a.y)) << 16);
    x.y = T::round(sum_once(T::lo(o.y), scale, a.z)) | (T::round(sum_once(T::hi(o.y), scale, a.w)) << 16);
    x.z = T::round(sum_once(T::lo(o.z), scale, b.x)) | (T::round(sum_once(T::hi(o.z), scale, b.y)) << 16);
    x.w = T::round(sum_once(T::lo(o.w), scale, b.z)) | (T::round(sum_once(T::hi(o.w), scale, b.w)) << 16);
    dst[c] = x;
  }
}

// pairs in sorted order: entry j comes from input position index[j]
__global__ void sort_pairs_gather_kernel(const uint32_t* __restrict__ index,
                                         const int32_t* __restrict__ centers,
                                         const int32_t* __restrict__ contexts, int64_t n,
                                         int32_t* __restrict__ centers_out,
                                         int32_t* __restrict__ contexts_out) {
  const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= n) return;
  const uint32_t from = index[j];
  centers_out[j] = centers[from];
  contexts_out[j] = contexts[from];
}

// ---- dense operations over a whole table: 16 bytes per lane, grid-stride ----------------
__global__ __launch_bounds__(256) void table_mult_f32_kernel(float4* __restrict__ t, int64_t n4,
                                                             float factor) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    float4 x = t[i];
    x.x *= factor; x.y *= factor; x.z *= factor; x.w *= factor;    // one exact product, rounded once
    t[i] = x;
  }
}
template <typename T>
__global__ __launch_bounds__(256) void table_mult16_kernel(uint4* __restrict__ t, int64_t n8,
                                                           float factor) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8;
       i += (int64_t)gridDim.x * blockDim.x) {
    uint4 x = t[i];
    x.x = T::round(T::lo(x.x) * factor) | (T::round(T::hi(x.x) * factor) << 16);
    x.y = T::round(T::lo(x.y) * factor) | (T::round(T::hi(x.y) * factor) << 16);
    x.z = T::round(T::lo(x.z) * factor) | (T::round(T::hi(x.z) * factor) << 16);
    x.w = T::round(T::lo(x.w) * factor) | (T::round(T::hi(x.w) * factor) << 16);
    t[i] = x;
  }
}
__global__ __launch_bounds__(256) void table_mult_add_f32_kernel(float4* __restrict__ dst,
                                                                 const float4* __restrict__ src,
                                                                 int64_t n4, float factor) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4;
       i += (int64_t)gridDim.x * blockDim.x) {
    const float4 o = dst[i], r = src[i];
    dst[i] = make_float4(sum_once(o.x, factor, r.x), sum_once(o.y, factor, r.y),
                         sum_once(o.z, factor, r.z), sum_once(o.w, factor, r.w));
  }
}
template <typename T>
__device__ __forceinline__ uint32_t mult_add_pair(uint32_t o, uint32_t r, float factor) {
  return T::round(sum_once(T::lo(o), factor, T::lo(r))) |
         (T::round(sum_once(T::hi(o), factor, T::hi(r))) << 16);
}
template <typename T>
__global__ __launch_bounds__(256) void table_mult_add16_kernel(uint4* __restrict__ dst,
                                                               const uint4* __restrict__ src,
                                                               int64_t n8, float factor) {
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n8;
       i += (int64_t)gridDim.x * blockDim.x) {
    const uint4 o = dst[i], r = src[i];
    uint4 x;
    x.x = mult_add_pair<T>(o.x, r.x, factor);
    x.y = mult_add_pair<T>(o.y, r.y, factor);
    x.z = mult_add_pair<T>(o.z, r.z, factor);
    x.w = mult_add_pair<T>(o.w, r.w, factor);
    dst[i] = x;
  }
}

int32_t check_table_args(const void* table, int64_t num_nodes, int32_t dim, int32_t dtype) {
  if (!table || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX) return GS_EINVAL;
  if (dtype != GS_F32 && dtype != GS_BF16 && dtype != GS_F16) return GS_EINVAL;
  if (dim < 1 || dim % (dtype == GS_F32 ? 4 : 8) != 0) return GS_EINVAL;
  if (!aligned(table, 16)) return GS_EINVAL;
  return GS_OK;
}

// The bitmap route costs a pass over num_nodes / 32 words, the sort route a few passes over the
// n ids: bitmap unless the graph is far larger than the batch.
bool unique_by_bitmap(int64_t n, int64_t num_nodes) { return ceil_div(num_nodes, 32) <= 8 * n; }

struct BitmapPlan {
  uint32_t* bitmap;
  int64_t *counts, *scan_scratch;
  int64_t words;
  size_t bytes;
};

BitmapPlan plan_bitmap(void* ws, int64_t num_nodes) {
  Carver cv(ws);
  BitmapPlan p;
  p.words = ceil_div(num_nodes > 0 ? num_nodes : 1, 32);
  p.bitmap = cv.take<uint32_t>((size_t)p.words);
  p.counts = cv.take<int64_t>((size_t)p.words);
  p.scan_scratch = cv.take<int64_t>(scan_scratch_elems(p.words));
  p.bytes = cv.used;
  return p;
}

struct UniquePlan {
  uint64_t *keys, *keys_alt;
  uint32_t *index, *index_alt;
  int64_t *head, *scan_scratch;
  void* sort_scratch;
  size_t bytes;
};

UniquePlan plan_unique(void* ws, int64_t n) {
  Carver cv(ws);
  UniquePlan p;
  const size_t m = (size_t)(n > 0 ? n : 1);
  p.keys = cv.take<uint64_t>(m);
  p.keys_alt = cv.take<uint64_t>(m);
  p.index = cv.take<uint32_t>(m);
  p.index_alt = cv.take<uint32_t>(m);
  p.head = cv.take<int64_t>(m);
  p.scan_scratch = cv.take<int64_t>(scan_scratch_elems((int64_t)m));
  p.sort_scratch = cv.take<char>(radix_sort_scratch_bytes((int64_t)m));
  p.bytes = cv.used;
  return p;
}

struct SortPairsPlan {
  uint64_t *keys, *keys_alt;
  uint32_t *index, *index_alt;
  void* sort_scratch;
  size_t bytes;
};

SortPairsPlan plan_sort_pairs(void* ws, int64_t n) {
  Carver cv(ws);
  SortPairsPlan p;
  const size_t m = (size_t)(n > 0 ? n : 1);
  p.keys = cv.take<uint64_t>(m);
  p.keys_alt = cv.take<uint64_t>(m);
  p.index = cv.take<uint32_t>(m);
  p.index_alt = cv.take<uint32_t>(m);
  p.sort_scratch = cv.take<char>(radix_sort_scratch_bytes((int64_t)m));
  p.bytes = cv.used;
  return p;
}

int bits_for(uint64_t max_value) {
  int b = 1;
  while (b < 64 && (max_value >> b) != 0) ++b;
  return b;
}

int32_t check_rows_args(const void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                        const int32_t* ids, int64_t n, const void* block) {
  if (!table || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX || n < 0) return GS_EINVAL;
  if (dtype != GS_F32 && dtype != GS_BF16 && dtype != GS_F16) return GS_EINVAL;
  if (dim < 1 || dim % (dtype == GS_F32 ? 4 : 8) != 0) return GS_EINVAL;
  if (n > 0 && (!ids || !block)) return GS_EINVAL;
  if (!aligned(table, 16) || (n > 0 && !aligned(block, 16))) return GS_EINVAL;
  if (ceil_div(n, kRowsPerBlock) > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  return GS_OK;
}

}  // namespace

}  // namespace gs

using namespace gs;

extern "C" size_t gs_unique_ids_workspace_bytes(int64_t n, int64_t num_nodes) {
  if (n < 0 || num_nodes < 1) return 0;
  if (unique_by_bitmap(n, num_nodes)) return plan_bitmap(nullptr, num_nodes).bytes;
  return plan_unique(nullptr, n).bytes;
}

extern "C" int32_t gs_unique_ids(const int32_t* ids, int64_t n, int64_t num_nodes, int32_t* unique_out,
                                 int64_t* num_unique_out, int32_t* inverse_out, void* ws,
                                 size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (n < 0 || n >= ((int64_t)1 << 31) || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX ||
      !num_unique_out)
    return GS_EINVAL;
  if (n > 0 && (!ids || !unique_out)) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  if (unique_by_bitmap(n, num_nodes)) {
    BitmapPlan b = plan_bitmap(ws, num_nodes);
    if (ws_bytes < b.bytes) return GS_EWORKSPACE;
    const unsigned word_blocks = (unsigned)ceil_div(b.words, 256);
    const unsigned id_blocks = (unsigned)ceil_div(n, 256);
    fill_words_kernel<<<word_blocks, 256, 0, stream>>>(b.bitmap, b.words, 0u);
    GS_LAUNCH_CHECK();
    bitmap_mark_kernel<<<id_blocks, 256, 0, stream>>>(ids, n, num_nodes, b.bitmap);
    GS_LAUNCH_CHECK();
    bitmap_count_kernel<<<word_blocks, 256, 0, stream>>>(b.bitmap, b.words, b.counts);
    GS_LAUNCH_CHECK();
    const int32_t rc = exclusive_scan_i64(b.counts, b.words, b.scan_scratch, num_unique_out, stream);
    if (rc != GS_OK) return rc;
    bitmap_emit_kernel<<<word_blocks, 256, 0, stream>>>(b.bitmap, b.counts, b.words, unique_out);
    GS_LAUNCH_CHECK();
    if (inverse_out) {
      bitmap_inverse_kernel<<<id_blocks, 256, 0, stream>>>(ids, n, num_nodes, b.bitmap, b.counts,
                                                          inverse_out);
      GS_LAUNCH_CHECK();
    }
    return GS_OK;
  }
  UniquePlan p = plan_unique(ws, n);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  const unsigned blocks = (unsigned)ceil_div(n, 256);
  if (n > 0) {
    unique_keys_kernel<<<blocks, 256, 0, stream>>>(ids, n, num_nodes, p.keys, p.index);
    GS_LAUNCH_CHECK();
    int32_t rc = radix_sort_u64_u32(p.keys, p.index, p.keys_alt, p.index_alt, n, 0,
                                    bits_for((uint64_t)num_nodes), 0, 0, p.sort_scratch, stream);
    if (rc != GS_OK) return rc;
    unique_heads_kernel<<<blocks, 256, 0, stream>>>(p.keys, n, num_nodes, p.head);
    GS_LAUNCH_CHECK();
  }
  int32_t rc = exclusive_scan_i64(p.head, n, p.scan_scratch, num_unique_out, stream);
  if (rc != GS_OK) return rc;
  if (n > 0) {
    unique_emit_kernel<<<blocks, 256, 0, stream>>>(p.keys, p.index, p.head, n, num_nodes, unique_out,
                                                   inverse_out);
    GS_LAUNCH_CHECK();
  }
  return GS_OK;
}

extern "C" int32_t gs_get_rows(const void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                               const int32_t* ids, int64_t n, const int64_t* count_dev, float* out,
                               void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t rc = check_rows_args(table, num_nodes, dim, dtype, ids, n, out);
  if (rc != GS_OK) return rc;
  if (n == 0) return GS_OK;
  const unsigned blocks = (unsigned)ceil_div(n, kRowsPerBlock);
  if (dtype == GS_F32)
    get_rows_f32_kernel<<<blocks, kRowThreads, 0, stream>>>(static_cast<const float*>(table), num_nodes,
                                                            dim, ids, n, count_dev, out);
  else if (dtype == GS_BF16)
    get_rows16_kernel<bf16_t><<<blocks, kRowThreads, 0, stream>>>(static_cast<const uint16_t*>(table),
                                                                  num_nodes, dim, ids, n, count_dev, out);
  else
    get_rows16_kernel<f16_t><<<blocks, kRowThreads, 0, stream>>>(static_cast<const uint16_t*>(table),
                                                                 num_nodes, dim, ids, n, count_dev, out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" int32_t gs_put_rows(void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                               const int32_t* ids, int64_t n, const int64_t* count_dev,
                               const float* rows, float scale, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t rc = check_rows_args(table, num_nodes, dim, dtype, ids, n, rows);
  if (rc != GS_OK) return rc;
  if (n == 0) return GS_OK;
  const unsigned blocks = (unsigned)ceil_div(n, kRowsPerBlock);
  if (dtype == GS_F32)
    put_rows_f32_kernel<<<blocks, kRowThreads, 0, stream>>>(static_cast<float*>(table), num_nodes, dim,
                                                            ids, n, count_dev, rows, scale);
  else if (dtype == GS_BF16)
    put_rows16_kernel<bf16_t><<<blocks, kRowThreads, 0, stream>>>(static_cast<uint16_t*>(table), num_nodes,
                                                                  dim, ids, n, count_dev, rows, scale);
  else
    put_rows16_kernel<f16_t><<<blocks, kRowThreads, 0, stream>>>(static_cast<uint16_t*>(table), num_nodes,
                                                                 dim, ids, n, count_dev, rows, scale);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" int32_t gs_table_mult(void* table, int64_t num_nodes, int32_t dim, int32_t dtype,
                                 float factor, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  const int32_t rc = check_table_args(table, num_nodes, dim, dtype);
  if (rc != GS_OK) return rc;
  const int64_t pieces = num_nodes * (int64_t)dim / (dtype == GS_F32 ? 4 : 8);
  const unsigned blocks = (unsigned)min((int64_t)(256 * 64), ceil_div(pieces, 256));
  if (dtype == GS_F32)
    table_mult_f32_kernel<<<blocks, 256, 0, stream>>>(static_cast<float4*>(table), pieces, factor);
  else if (dtype == GS_BF16)
    table_mult16_kernel<bf16_t><<<blocks, 256, 0, stream>>>(static_cast<uint4*>(table), pieces, factor);
  else
    table_mult16_kernel<f16_t><<<blocks, 256, 0, stream>>>(static_cast<uint4*>(table), pieces, factor);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" int32_t gs_table_mult_add(void* dst, const void* src, int64_t num_nodes, int32_t dim,
                                     int32_t dtype, float factor, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  int32_t rc = check_table_args(dst, num_nodes, dim, dtype);
  if (rc != GS_OK) return rc;
  rc = check_table_args(src, num_nodes, dim, dtype);
  if (rc != GS_OK) return rc;
  if (dst == src) return GS_EINVAL;
  const int64_t pieces = num_nodes * (int64_t)dim / (dtype == GS_F32 ? 4 : 8);
  const unsigned blocks = (unsigned)min((int64_t)(256 * 64), ceil_div(pieces, 256));
  if (dtype == GS_F32)
    table_mult_add_f32_kernel<<<blocks, 256, 0, stream>>>(static_cast<float4*>(dst),
                                                          static_cast<const float4*>(src), pieces, factor);
  else if (dtype == GS_BF16)
    table_mult_add16_kernel<bf16_t><<<blocks, 256, 0, stream>>>(
        static_cast<uint4*>(dst), static_cast<const uint4*>(src), pieces, factor);
  else
    table_mult_add16_kernel<f16_t><<<blocks, 256, 0, stream>>>(
        static_cast<uint4*>(dst), static_cast<const uint4*>(src), pieces, factor);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" size_t gs_sort_pairs_workspace_bytes(int64_t n) {
  if (n < 0) return 0;
  return plan_sort_pairs(nullptr, n).bytes;
}

extern "C" int32_t gs_sort_pairs(const int32_t* centers, const int32_t* contexts, int64_t n,
                                 int64_t num_nodes, int32_t* centers_out, int32_t* contexts_out,
                                 void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (n < 0 || n >= ((int64_t)1 << 31) || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX)
    return GS_EINVAL;
  if (n > 0 && (!centers || !contexts || !centers_out || !contexts_out)) return GS_EINVAL;
  if (n > 0 && (centers_out == centers || contexts_out == contexts)) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  SortPairsPlan p = plan_sort_pairs(ws, n);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  if (n == 0) return GS_OK;
  const unsigned blocks = (unsigned)ceil_div(n, 256);
  unique_keys_kernel<<<blocks, 256, 0, stream>>>(centers, n, num_nodes, p.keys, p.index);
  GS_LAUNCH_CHECK();
  const int32_t rc = radix_sort_u64_u32(p.keys, p.index, p.keys_alt, p.index_alt, n, 0,
                                        bits_for((uint64_t)num_nodes), 0, 0, p.sort_scratch, stream);
  if (rc != GS_OK) return rc;
  sort_pairs_gather_kernel<<<blocks, 256, 0, stream>>>(p.index, centers, contexts, n, centers_out,
                                                       contexts_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
