// gs_make_pairs and gs_sample_negatives (GraphScale Sec. 2.2: skip-gram with
// negative sampling over the walks; Sec. 3.2: the positively and negatively
// sampled nodes of a batch).
#include "common.h"

namespace gs {

__global__ void pairs_count_kernel(const int32_t* __restrict__ walks, int64_t num_walks,
                                   int32_t walk_len, int32_t window, int64_t* __restrict__ counts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_walks) return;
  const int32_t len = valid_prefix(walks + i * (int64_t)walk_len, walk_len);
  counts[i] = 2 * window_prefix(len, window);
}

constexpr int kEmitThreads = 256;
constexpr int kEmitLdsInts = 10240;   // staged walk window: walks_per_block * walk_len <= this
constexpr int kEmitMaxWalks = 64;

__global__ __launch_bounds__(kEmitThreads) void pairs_emit_kernel(
    const int32_t* __restrict__ walks, int64_t num_walks, int32_t walk_len, int32_t window,
    int walks_per_block, const int64_t* __restrict__ bases, const int64_t* __restrict__ total,
    int32_t* __restrict__ centers, int32_t* __restrict__ contexts) {
  __shared__ int32_t rows[kEmitLdsInts];
  __shared__ int64_t base_s[kEmitMaxWalks + 1];
  __shared__ int32_t len_s[kEmitMaxWalks];
  const int64_t w0 = (int64_t)blockIdx.x * walks_per_block;
  const int g_count = (int)min((int64_t)walks_per_block, num_walks - w0);
  const int64_t ints = (int64_t)g_count * walk_len;
  const int32_t* src = walks + w0 * (int64_t)walk_len;
  for (int64_t x = threadIdx.x; x < ints; x += kEmitThreads) rows[x] = src[x];
  for (int g = threadIdx.x; g <= g_count; g += kEmitThreads)
    base_s[g] = (w0 + g < num_walks) ? bases[w0 + g] : *total;
  __syncthreads();
  for (int g = threadIdx.x; g < g_count; g += kEmitThreads)
    len_s[g] = valid_prefix(rows + g * walk_len, walk_len);
  __syncthreads();
  const int64_t first = base_s[0], last = base_s[g_count];
  for (int64_t p = first + threadIdx.x; p < last; p += kEmitThreads) {
    // walk of this pair: last g with base_s[g] <= p
    int lo = 0, hi = g_count - 1;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (base_s[mid] <= p) lo = mid; else hi = mid - 1;
    }
    const int g = lo;
    const int64_t q = p - base_s[g];
    const int64_t len = len_s[g];
    int64_t a, other;
    pair_positions(q, len, window, a, other);
    const int32_t* row = rows + g * walk_len;
    centers[p] = row[a];
    contexts[p] = row[other];
  }
}

__global__ void negatives_kernel(const float* __restrict__ prob, const int32_t* __restrict__ alias,
                                 const uint2* __restrict__ packed,
                                 uint64_t num_nodes, int64_t total, uint64_t pair_base, int32_t k,
                                 uint64_t seed, int32_t* __restrict__ negs) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= total) return;
  const uint64_t i = (uint64_t)(e / k);
  const uint32_t j = (uint32_t)(e - (int64_t)i * k);
  const Block4 b = philox_at(seed, pair_base + i, j, 0x80000000u);
  negs[e] = (int32_t)table_draw(prob, alias, packed, num_nodes, b);
}

// One lane per LINE sample: draw an entry, then find the row that holds it
// (the last row whose offset is <= e; empty rows share their offset with the
// next row and are skipped by taking the last one).
template <typename OffT>
__global__ void edges_kernel(const OffT* __restrict__ offsets, int64_t num_nodes,
                             const int32_t* __restrict__ nbrs, uint64_t num_entries,
                             const float* __restrict__ prob, const int32_t* __restrict__ alias,
                             const uint2* __restrict__ packed, int64_t num_samples,
                             uint64_t sample_base, uint64_t seed, int32_t* __restrict__ centers,
                             int32_t* __restrict__ contexts) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= num_samples) return;
  const Block4 b = philox_at(seed, sample_base + (uint64_t)i, 0u, 0x40000000u);
  const int64_t e = table_draw(prob, alias, packed, num_entries, b);
  const int32_t dst = nbrs[e];
  // first t in [1, num_nodes] with offsets[t] > e; offsets[num_nodes] = num_entries > e
  int64_t lo = 1, hi = num_nodes;
  while (lo < hi) {
    const int64_t mid = (lo + hi) >> 1;
    if ((int64_t)offsets[mid] > e) hi = mid; else lo = mid + 1;
  }
  centers[i] = (int32_t)(lo - 1);
  contexts[i] = dst;
}

struct PairsPlan {
  int64_t *bases, *scan_scratch;
  size_t bytes;
};
static PairsPlan plan_pairs(void* ws, int64_t num_walks) {
  Carver cv(ws);
  PairsPlan p;
  const size_t n = (size_t)(num_walks > 0 ? num_walks : 1);
  p.bases = cv.take<int64_t>(n);
  p.scan_scratch = cv.take<int64_t>(scan_scratch_elems((int64_t)n));
  p.bytes = cv.used;
  return p;
}

}  // namespace gs

using namespace gs;

extern "C" size_t gs_make_pairs_workspace_bytes(int64_t num_walks) {
  if (num_walks < 0) return 0;
  return plan_pairs(nullptr, num_walks).bytes;
}

extern "C" int32_t gs_make_pairs(const int32_t* walks, int64_t num_walks, int32_t walk_len,
                                 int32_t window, int32_t* centers_out, int32_t* contexts_out,
                                 int64_t* num_pairs_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (num_walks < 0 || walk_len < 1 || walk_len > 4096 || window < 1 || !num_pairs_out)
    return GS_EINVAL;
  if (num_walks > 0 && !walks) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  PairsPlan p = plan_pairs(ws, num_walks);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  const bool may_emit = walk_len > 1;
  if (num_walks > 0 && may_emit && (!centers_out || !contexts_out)) return GS_EINVAL;
  if (num_walks > 0) {
    pairs_count_kernel<<<(unsigned)ceil_div(num_walks, 256), 256, 0, stream>>>(walks, num_walks, walk_len,
                                                                             window, p.bases);
    GS_LAUNCH_CHECK();
  }
  int32_t rc = exclusive_scan_i64(p.bases, num_walks, p.scan_scratch, num_pairs_out, stream);
  if (rc != GS_OK) return rc;
  if (num_walks > 0 && may_emit) {
    int wpb = kEmitLdsInts / walk_len;
    if (wpb > kEmitMaxWalks) wpb = kEmitMaxWalks;
    if (wpb < 1) wpb = 1;
    pairs_emit_kernel<<<(unsigned)ceil_div(num_walks, wpb), kEmitThreads, 0, stream>>>(
        walks, num_walks, walk_len, window, wpb, p.bases, num_pairs_out, centers_out, contexts_out);
    GS_LAUNCH_CHECK();
  }
  return GS_OK;
}

extern "C" size_t gs_pair_offsets_workspace_bytes(int64_t num_walks) {
  if (num_walks < 0) return 0;
  Carver cv(nullptr);
  cv.take<int64_t>(scan_scratch_elems(num_walks > 0 ? num_walks : 1));
  return cv.used;
}

extern "C" int32_t gs_pair_offsets(const int32_t* walks, int64_t num_walks, int32_t walk_len,
                                   int32_t window, int64_t* offsets_out, void* ws, size_t ws_bytes,
                                   void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (num_walks < 0 || walk_len < 1 || walk_len > 4096 || window < 1 || !offsets_out) return GS_EINVAL;
  if (num_walks > 0 && !walks) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  if (ws_bytes < gs_pair_offsets_workspace_bytes(num_walks)) return GS_EWORKSPACE;
  if (num_walks > 0) {
    pairs_count_kernel<<<(unsigned)ceil_div(num_walks, 256), 256, 0, stream>>>(walks, num_walks, walk_len,
                                                                             window, offsets_out);
    GS_LAUNCH_CHECK();
  }
  // exclusive sums in place; the total goes to the entry after the last walk
  return exclusive_scan_i64(offsets_out, num_walks, static_cast<int64_t*>(ws), offsets_out + num_walks,
                            stream);
}

extern "C" int32_t gs_sample_negatives(const gs_alias* noise, int64_t num_nodes, int64_t num_pairs,
                                       uint64_t pair_index_base, int32_t k, uint64_t seed,
                                       int32_t* negs_out, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (num_nodes < 1 || num_nodes > (int64_t)INT32_MAX || num_pairs < 0 || k < 0) return GS_EINVAL;
  if (num_pairs > 0 && k > 0 && !negs_out) return GS_EINVAL;
  const bool weighted = noise != nullptr && noise->prob != nullptr;
  if (weighted && !noise->alias) return GS_EINVAL;
  const int64_t total = num_pairs * (int64_t)k;
  if (total == 0) return GS_OK;
  if (ceil_div(total, 256) > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  negatives_kernel<<<(unsigned)ceil_div(total, 256), 256, 0, stream>>>(
      weighted ? noise->prob : nullptr, weighted ? noise->alias : nullptr,
      weighted ? reinterpret_cast<const uint2*>(noise->packed) : nullptr, (uint64_t)num_nodes, total,
      pair_index_base, k, seed, negs_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

extern "C" int32_t gs_sample_edges(const gs_csr* g, const gs_alias* edge_alias, int64_t num_samples,
                                   uint64_t sample_index_base, uint64_t seed, int32_t* centers_out,
                                   int32_t* contexts_out, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!g || g->num_nodes < 1 || g->num_nodes > (int64_t)INT32_MAX || g->num_entries < 1 ||
      !g->offsets || !g->nbrs || num_samples < 0)
    return GS_EINVAL;
  if (g->offset_bits != 32 && g->offset_bits != 64) return GS_EINVAL;
  if (num_samples > 0 && (!centers_out || !contexts_out)) return GS_EINVAL;
  const bool weighted = edge_alias != nullptr && edge_alias->prob != nullptr;
  if (weighted && !edge_alias->alias) return GS_EINVAL;
  if (num_samples == 0) return GS_OK;
  if (ceil_div(num_samples, 256) > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  const float* prob = weighted ? edge_alias->prob : nullptr;
  const int32_t* alias = weighted ? edge_alias->alias : nullptr;
  const uint2* packed = weighted ? reinterpret_cast<const uint2*>(edge_alias->packed) : nullptr;
  const unsigned blocks = (unsigned)ceil_div(num_samples, 256);
  if (g->offset_bits == 32)
    edges_kernel<int32_t><<<blocks, 256, 0, stream>>>(
        static_cast<const int32_t*>(g->offsets), g->num_nodes, g->nbrs, (uint64_t)g->num_entries, prob,
        alias, packed, num_samples, sample_index_base, seed, centers_out, contexts_out);
  else
    edges_kernel<int64_t><<<blocks, 256, 0, stream>>>(
        static_cast<const int64_t*>(g->offsets), g->num_nodes, g->nbrs, (uint64_t)g->num_entries, prob,
        alias, packed, num_samples, sample_index_base, seed, centers_out, contexts_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
