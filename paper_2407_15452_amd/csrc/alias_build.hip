// gs_alias_build: alias tables, one per segment, in the canonical first-in
// first-out construction order stated in gs.h (Walker 1977 / Vose 1991).
// The order of the fp64 operations is part of the definition of the table, so
// each segment is built sequentially by one lane; parallelism is across
// segments (per-row tables of a weighted graph).
#include "common.h"

namespace gs {

template <typename OffT>
__global__ __launch_bounds__(64) void alias_build_kernel(const OffT* __restrict__ seg_offsets,
                                                         int64_t num_segments,
                                                         const float* __restrict__ weights,
                                                         float* __restrict__ prob_out,
                                                         int32_t* __restrict__ alias_out,
                                                         double* __restrict__ mass_ws,
                                                         int32_t* __restrict__ small_ws,
                                                         int32_t* __restrict__ large_ws) {
#pragma clang fp contract(off)  // every fp64 operation below must round on its own
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= num_segments) return;
  const int64_t begin = (int64_t)seg_offsets[s];
  const int64_t n = (int64_t)seg_offsets[s + 1] - begin;
  if (n <= 0) return;
  const float* w = weights + begin;
  float* prob = prob_out + begin;
  int32_t* alias = alias_out + begin;
  double* mass = mass_ws + begin;
  int32_t* small_q = small_ws + begin;   // every entry enters at most once: no wrap
  int32_t* large_q = large_ws + begin;   // ring of capacity n

  double S = 0.0;
  for (int64_t i = 0; i < n; ++i) S += (double)w[i];
  int64_t small_head = 0, small_tail = 0;
  int64_t large_head = 0, large_count = 0;
  const double dn = (double)n;
  for (int64_t i = 0; i < n; ++i) {
    const double m = (double)w[i] * dn;
    mass[i] = m;
    if (m < S) small_q[small_tail++] = (int32_t)i;
    else large_q[large_count++] = (int32_t)i;
  }
  while (small_head < small_tail && large_count > 0) {
    const int32_t a = small_q[small_head++];
    const int32_t b = large_q[large_head];
    large_head = (large_head + 1 == n) ? 0 : large_head + 1;
    --large_count;
    const double ma = mass[a];
    prob[a] = (float)(ma / S);
    alias[a] = b;
    const double mb = (mass[b] + ma) - S;
    mass[b] = mb;
    if (mb < S) {
      small_q[small_tail++] = b;
    } else {
      int64_t at = large_head + large_count;
      if (at >= n) at -= n;
      large_q[at] = b;
      ++large_count;
    }
  }
  for (; small_head < small_tail; ++small_head) {
    const int32_t i = small_q[small_head];
    prob[i] = 1.0f;
    alias[i] = i;
  }
  for (; large_count > 0; --large_count) {
    const int32_t i = large_q[large_head];
    large_head = (large_head + 1 == n) ? 0 : large_head + 1;
    prob[i] = 1.0f;
    alias[i] = i;
  }
}

struct AliasPlan {
  double* mass;
  int32_t *small_q, *large_q;
  size_t bytes;
};

static AliasPlan plan_alias(void* ws, int64_t total_entries) {
  Carver cv(ws);
  AliasPlan p;
  const size_t t = (size_t)(total_entries > 0 ? total_entries : 1);
  p.mass = cv.take<double>(t);
  p.small_q = cv.take<int32_t>(t);
  p.large_q = cv.take<int32_t>(t);
  p.bytes = cv.used;
  return p;
}

}  // namespace gs

using namespace gs;

extern "C" size_t gs_alias_build_workspace_bytes(int64_t num_segments, int64_t total_entries) {
  (void)num_segments;
  if (total_entries < 0) return 0;
  return plan_alias(nullptr, total_entries).bytes;
}

extern "C" int32_t gs_alias_build(const void* seg_offsets, int32_t offset_bits, int64_t num_segments,
                                  int64_t total_entries, const float* weights, float* prob_out,
                                  int32_t* alias_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (offset_bits != 32 && offset_bits != 64) return GS_EINVAL;
  if (num_segments < 0 || total_entries < 0 || !seg_offsets) return GS_EINVAL;
  if (total_entries > 0 && (!weights || !prob_out || !alias_out)) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  AliasPlan p = plan_alias(ws, total_entries);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  if (num_segments == 0 || total_entries == 0) return GS_OK;
  const int threads = 64;
  const unsigned blocks = (unsigned)ceil_div(num_segments, threads);
  if (offset_bits == 64)
    alias_build_kernel<int64_t><<<blocks, threads, 0, stream>>>((const int64_t*)seg_offsets,
        num_segments, weights, prob_out, alias_out, p.mass, p.small_q, p.large_q);
  else
    alias_build_kernel<int32_t><<<blocks, threads, 0, stream>>>((const int32_t*)seg_offsets,
        num_segments, weights, prob_out, alias_out, p.mass, p.small_q, p.large_q);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
