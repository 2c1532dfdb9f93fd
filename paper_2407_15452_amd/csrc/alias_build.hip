// gs_alias_build: alias tables, one per segment, in the canonical first-in
// first-out construction order stated in gs.h (Walker 1977 / Vose 1991).
// The order of the fp64 operations is part of the definition of the table, so
// each short segment is built sequentially by one lane; parallelism is across
// segments (per-row tables of a weighted graph).  Long segments (the noise
// table, the rows of hub nodes) are built by one workgroup each, see
// alias_build_long_kernel.
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
                                                         int32_t* __restrict__ large_ws,
                                                         int64_t skip_from) {
#pragma clang fp contract(off)  // every fp64 operation below must round on its own
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= num_segments) return;
  const int64_t begin = (int64_t)seg_offsets[s];
  const int64_t n = (int64_t)seg_offsets[s + 1] - begin;
  if (n <= 0 || n >= skip_from) return;        // long segments are left to the workgroup kernel
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

// ---------------------------------------------------------------------------
// A long segment (the noise table, a hub row): the same construction, same order,
// run by one workgroup of 1024 lanes.
//
// The sequential loop pairs the oldest small with the oldest large and appends
// the large to the back of one of the two lists.  If both lists hold at least m
// entries, the next m iterations use exactly the first m entries of each list
// as they stand now (appends go to the back), touch 2m distinct entries, and
// are independent of each other: they can run side by side, and appending
// their larges in iteration order (a prefix sum over the "became small" flags)
// leaves both lists exactly as the sequential loop would.  So the workgroup
// advances in rounds of m = min(|small|, |large|) iterations; when m is small
// (a few very heavy entries left) lane 0 runs the plain loop instead.
// S is still the index-order fp64 sum: lanes stage 1024 weights in LDS, lane 0
// adds them one by one.
// ---------------------------------------------------------------------------
constexpr int kLongThreads = 1024;
constexpr int64_t kLongSegment = 8192;      // segments at least this long use the workgroup
constexpr int kSerialBelow = 64;            // rounds narrower than this are run by lane 0

// loads that must see what other lanes of the workgroup stored earlier (bypass the L1)
__device__ __forceinline__ int32_t ld_i32(const int32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ double ld_f64(const double* p) {
  return __longlong_as_double((long long)__hip_atomic_load(
      reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
}

// Ranks of the set flags among the 1024 lanes, in lane order, and their total.
__device__ __forceinline__ void block_rank(bool flag, uint32_t* wave_tot, int& rank, int& total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t votes = __ballot(flag);
  const int before = __popcll(votes & ((1ull << lane) - 1ull));
  if (lane == 0) wave_tot[wave] = (uint32_t)__popcll(votes);
  __syncthreads();
  int base = 0, all = 0;
#pragma unroll
  for (int w = 0; w < kLongThreads / 64; ++w) {
    const int c = (int)wave_tot[w];
    if (w < wave) base += c;
    all += c;
  }
  __syncthreads();
  rank = base + before;
  total = all;
}

// the segments the workgroup kernel takes, in any order
template <typename OffT>
__global__ void alias_find_long_kernel(const OffT* __restrict__ seg_offsets, int64_t num_segments,
                                       int64_t* __restrict__ long_ids, int64_t capacity,
                                       unsigned long long* __restrict__ long_count) {
  const int64_t s = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= num_segments) return;
  if ((int64_t)seg_offsets[s + 1] - (int64_t)seg_offsets[s] >= kLongSegment) {
    // capacity = total_entries / kLongSegment bounds the count when the offsets add up to
    // total_entries; an inconsistent pair of arguments must still not write out of bounds
    const unsigned long long at = atomicAdd(long_count, 1ull);
    if (at < (unsigned long long)capacity) long_ids[at] = s;
  }
}

__global__ void zero_u64_kernel(unsigned long long* p) { *p = 0ull; }

// One workgroup per long segment.  long_ids == null: the single segment 0.
// Scratch per entry of the segment, at the segment's own offsets: mass, the
// small list (n entries), the large list (2n: appended without wrapping).
template <typename OffT>
__global__ __launch_bounds__(kLongThreads) void alias_build_long_kernel(
    const OffT* __restrict__ seg_offsets, const int64_t* __restrict__ long_ids,
    const unsigned long long* __restrict__ long_count, const float* __restrict__ weights,
    float* __restrict__ prob_out, int32_t* __restrict__ alias_out, double* mass_ws,
    int32_t* small_ws, int32_t* large_ws) {
#pragma clang fp contract(off)  // every fp64 operation below must round on its own
  __shared__ double tile_s[kLongThreads];
  __shared__ uint32_t wave_tot[kLongThreads / 64];
  __shared__ double S_s;
  __shared__ int64_t q_s[4];                  // small head/tail, large head/tail after a serial stretch
  const int tid = threadIdx.x;
  if (long_ids != nullptr && (unsigned long long)blockIdx.x >= *long_count) return;
  const int64_t seg = long_ids != nullptr ? long_ids[blockIdx.x] : 0;
  const int64_t begin = (int64_t)seg_offsets[seg];
  const int64_t n = (int64_t)seg_offsets[seg + 1] - begin;
  if (n <= 0) return;
  const float* w = weights + begin;
  float* prob = prob_out + begin;
  int32_t* alias = alias_out + begin;
  double* mass = mass_ws + begin;
  int32_t* small_q = small_ws + begin;
  int32_t* large_q = large_ws + 2 * begin;

  // S: index-order sum
  double run = 0.0;
  for (int64_t base = 0; base < n; base += kLongThreads) {
    tile_s[tid] = (base + tid < n) ? (double)w[base + tid] : 0.0;
    __syncthreads();
    if (tid == 0) {
      const int cnt = (int)min((int64_t)kLongThreads, n - base);
      for (int k = 0; k < cnt; ++k) run += tile_s[k];
    }
    __syncthreads();
  }
  if (tid == 0) S_s = run;
  __syncthreads();
  const double S = S_s;
  const double dn = (double)n;

  // initial lists, in index order
  int64_t sh = 0, st = 0, lh = 0, lt = 0;     // heads and tails, identical in every lane
  for (int64_t base = 0; base < n; base += kLongThreads) {
    const int64_t i = base + tid;
    const bool valid = i < n;
    double m = 0.0;
    if (valid) { m = (double)w[i] * dn; mass[i] = m; }
    const bool is_small = valid && m < S;
    int rs, ts, rl, tl;
    block_rank(is_small, wave_tot, rs, ts);
    block_rank(valid && !is_small, wave_tot, rl, tl);
    if (is_small) small_q[st + rs] = (int32_t)i;
    else if (valid) large_q[lt + rl] = (int32_t)i;
    st += ts;
    lt += tl;
  }

  while (true) {
    __threadfence();
    __syncthreads();
    const int64_t m = min(st - sh, lt - lh);
    if (m <= 0) break;
    if (m < kSerialBelow) {
      // few entries on one side: the plain loop, for a bounded stretch
      if (tid == 0) {
        int64_t a_sh = sh, a_st = st, a_lh = lh, a_lt = lt;
        for (int it = 0; it < 4096 && a_sh < a_st && a_lh < a_lt; ++it) {
          const int32_t a = ld_i32(small_q + a_sh++);
          const int32_t b = ld_i32(large_q + a_lh++);
          const double ma = ld_f64(mass + a);
          prob[a] = (float)(ma / S);
          alias[a] = b;
          const double mb = (ld_f64(mass + b) + ma) - S;
          mass[b] = mb;
          if (mb < S) small_q[a_st++] = b; else large_q[a_lt++] = b;
        }
        q_s[0] = a_sh; q_s[1] = a_st; q_s[2] = a_lh; q_s[3] = a_lt;
      }
      __syncthreads();
      sh = q_s[0]; st = q_s[1]; lh = q_s[2]; lt = q_s[3];
      continue;
    }
    int64_t add_s = 0, add_l = 0;
    for (int64_t base = 0; base < m; base += kLongThreads) {
      const int64_t i = base + tid;
      const bool valid = i < m;
      int32_t b = 0;
      bool demoted = false;
      if (valid) {
        const int32_t a = ld_i32(small_q + sh + i);
        b = ld_i32(large_q + lh + i);
        const double ma = ld_f64(mass + a);
        prob[a] = (float)(ma / S);
        alias[a] = b;
        const double mb = (ld_f64(mass + b) + ma) - S;
        mass[b] = mb;
        demoted = mb < S;
      }
      int rs, ts, rl, tl;
      block_rank(valid && demoted, wave_tot, rs, ts);
      block_rank(valid && !demoted, wave_tot, rl, tl);
      if (valid) {
        if (demoted) small_q[st + add_s + rs] = b;
        else large_q[lt + add_l + rl] = b;
      }
      add_s += ts;
      add_l += tl;
    }
    sh += m; lh += m;
    st += add_s; lt += add_l;
  }
  for (int64_t i = sh + tid; i < st; i += kLongThreads) {
    const int32_t x = ld_i32(small_q + i);
    prob[x] = 1.0f; alias[x] = x;
  }
  for (int64_t i = lh + tid; i < lt; i += kLongThreads) {
    const int32_t x = ld_i32(large_q + i);
    prob[x] = 1.0f; alias[x] = x;
  }
}

__global__ void alias_pack_kernel(const float* __restrict__ prob, const int32_t* __restrict__ alias,
                                  int64_t n, uint64_t* __restrict__ packed) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) packed[i] = ((uint64_t)(uint32_t)alias[i] << 32) | (uint64_t)__float_as_uint(prob[i]);
}

struct AliasPlan {
  double* mass;
  int32_t *small_q, *large_q;
  int64_t* long_ids;
  unsigned long long* long_count;
  int64_t max_long;
  size_t bytes;
};

static AliasPlan plan_alias(void* ws, int64_t total_entries) {
  Carver cv(ws);
  AliasPlan p;
  const size_t t = (size_t)(total_entries > 0 ? total_entries : 1);
  p.mass = cv.take<double>(t);
  p.small_q = cv.take<int32_t>(t);
  p.large_q = cv.take<int32_t>(2 * t);   // the workgroup variant appends without wrapping
  p.max_long = (int64_t)(t / (size_t)kLongSegment) + 1;
  p.long_ids = cv.take<int64_t>((size_t)p.max_long);
  p.long_count = cv.take<unsigned long long>(1);
  p.bytes = cv.used;
  return p;
}

template <typename OffT>
static int32_t launch_alias_build(const OffT* seg_offsets, int64_t num_segments, int64_t total_entries,
                                  const float* weights, float* prob_out, int32_t* alias_out,
                                  const AliasPlan& p, hipStream_t stream) {
  if (num_segments == 1) {
    if (total_entries >= kLongSegment) {
      alias_build_long_kernel<OffT><<<1, kLongThreads, 0, stream>>>(
          seg_offsets, nullptr, nullptr, weights, prob_out, alias_out, p.mass, p.small_q, p.large_q);
      GS_LAUNCH_CHECK();
      return GS_OK;
    }
  }
  const int threads = 64;
  const unsigned blocks = (unsigned)ceil_div(num_segments, threads);
  // at most this many segments can be long; none: the lane kernel alone
  const int64_t max_long = min(num_segments, total_entries / kLongSegment);
  alias_build_kernel<OffT><<<blocks, threads, 0, stream>>>(
      seg_offsets, num_segments, weights, prob_out, alias_out, p.mass, p.small_q, p.large_q,
      max_long > 0 ? kLongSegment : INT64_MAX);
  GS_LAUNCH_CHECK();
  if (max_long > 0) {
    zero_u64_kernel<<<1, 1, 0, stream>>>(p.long_count);
    GS_LAUNCH_CHECK();
    alias_find_long_kernel<OffT><<<(unsigned)ceil_div(num_segments, 256), 256, 0, stream>>>(
        seg_offsets, num_segments, p.long_ids, max_long, p.long_count);
    GS_LAUNCH_CHECK();
    alias_build_long_kernel<OffT><<<(unsigned)max_long, kLongThreads, 0, stream>>>(
        seg_offsets, p.long_ids, p.long_count, weights, prob_out, alias_out, p.mass, p.small_q,
        p.large_q);
    GS_LAUNCH_CHECK();
  }
  return GS_OK;
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
  // alias[] holds 32-bit positions inside a segment; one segment over everything is the
  // one case the host can see
  if (num_segments == 1 && total_entries > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  if (num_segments == 0 || total_entries == 0) return GS_OK;
  if (offset_bits == 64)
    return launch_alias_build((const int64_t*)seg_offsets, num_segments, total_entries, weights,
                              prob_out, alias_out, p, stream);
  return launch_alias_build((const int32_t*)seg_offsets, num_segments, total_entries, weights, prob_out,
                            alias_out, p, stream);
}

extern "C" int32_t gs_alias_pack(const float* prob, const int32_t* alias, int64_t total_entries,
                                 uint64_t* packed_out, void* stream_) {
  if (total_entries < 0) return GS_EINVAL;
  if (total_entries == 0) return GS_OK;
  if (!prob || !alias || !packed_out || !aligned(packed_out, 8)) return GS_EINVAL;
  alias_pack_kernel<<<(unsigned)ceil_div(total_entries, 256), 256, 0, (hipStream_t)stream_>>>(
      prob, alias, total_entries, packed_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
