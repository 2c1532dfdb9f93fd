// Device-wide exclusive scan and a stable LSD radix sort (setup-side helpers of
// CSR construction and pair emission).
#include "common.h"

namespace gs {

static thread_local hipError_t g_last_error = hipSuccess;
void set_last_hip_error(hipError_t e) { g_last_error = e; }

extern "C" int32_t gs_last_hip_error(void) { return (int32_t)g_last_error; }

// ---------------------------------------------------------------------------
// Exclusive scan: tiles of 1024 values, tile totals scanned recursively.
// ---------------------------------------------------------------------------
constexpr int kScanThreads = 256;
constexpr int kScanItems = 4;
constexpr int kScanTile = kScanThreads * kScanItems;

__global__ __launch_bounds__(kScanThreads) void scan_tiles_kernel(int64_t* __restrict__ data,
                                                                  int64_t n,
                                                                  int64_t* __restrict__ tile_sums) {
  __shared__ int64_t wave_sums[kScanThreads / 64];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
  int64_t v[kScanItems];
  int64_t local = 0;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    v[k] = (base + k < n) ? data[base + k] : 0;
    local += v[k];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int64_t incl = local;
#pragma unroll
  for (int d = 1; d < 64; d <<= 1) {
    int64_t up = __shfl_up(incl, d, 64);
    if (lane >= d) incl += up;
  }
  if (lane == 63) wave_sums[wave] = incl;
  __syncthreads();
  int64_t wave_base = 0, total = 0;
#pragma unroll
  for (int w = 0; w < kScanThreads / 64; ++w) {
    if (w < wave) wave_base += wave_sums[w];
    total += wave_sums[w];
  }
  int64_t run = wave_base + incl - local;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k) {
    if (base + k < n) data[base + k] = run;
    run += v[k];
  }
  if (threadIdx.x == 0) tile_sums[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void scan_add_kernel(int64_t* __restrict__ data, int64_t n,
                                                                const int64_t* __restrict__ tile_offsets) {
  const int64_t add = tile_offsets[blockIdx.x];
  const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
#pragma unroll
  for (int k = 0; k < kScanItems; ++k)
    if (base + k < n) data[base + k] += add;
}

__global__ void copy_one_i64_kernel(const int64_t* src, int64_t* dst) { *dst = src ? *src : 0; }

size_t scan_scratch_elems(int64_t n) {
  size_t total = 1;
  while (n > 1) {
    n = ceil_div(n, kScanTile);
    total += (size_t)n;
    if (n == 1) break;
  }
  return total + 1;
}

int32_t exclusive_scan_i64(int64_t* data, int64_t n, int64_t* scratch, int64_t* total_out,
                           hipStream_t stream) {
  if (n <= 0) {
    if (total_out) {
      copy_one_i64_kernel<<<1, 1, 0, stream>>>(nullptr, total_out);
      GS_LAUNCH_CHECK();
    }
    return GS_OK;
  }
  constexpr int kMaxLevels = 8;
  int64_t* ptr[kMaxLevels + 1];
  int64_t size[kMaxLevels + 1];
  ptr[0] = data;
  size[0] = n;
  int levels = 0;
  size_t used = 0;
  while (true) {
    const int64_t tiles = ceil_div(size[levels], kScanTile);
    ptr[levels + 1] = scratch + used;
    size[levels + 1] = tiles;
    used += (size_t)tiles;
    scan_tiles_kernel<<<dim3((unsigned)tiles), kScanThreads, 0, stream>>>(ptr[levels], size[levels],
                                                                           ptr[levels + 1]);
    GS_LAUNCH_CHECK();
    ++levels;
    if (tiles == 1 || levels == kMaxLevels) break;
  }
  // ptr[levels][0] is the grand total (single tile at the top level)
  if (total_out) {
    copy_one_i64_kernel<<<1, 1, 0, stream>>>(ptr[levels], total_out);
    GS_LAUNCH_CHECK();
  }
  for (int l = levels - 2; l >= 0; --l) {
    scan_add_kernel<<<dim3((unsigned)size[l + 1]), kScanThreads, 0, stream>>>(ptr[l], size[l],
                                                                               ptr[l + 1]);
    GS_LAUNCH_CHECK();
  }
  return GS_OK;
}

// ---------------------------------------------------------------------------
// Radix sort.  One wave per tile of 2048 records; records of a tile are taken
// 64 at a time in index order, so ranking records of equal digit by (chunk,
// lane) keeps the sort stable.
// ---------------------------------------------------------------------------
constexpr int kSortItems = 32;
constexpr int kSortTile = 64 * kSortItems;
constexpr int kMaxDigitBits = 8;

__global__ __launch_bounds__(64) void radix_hist_kernel(const uint64_t* __restrict__ keys, int64_t n,
                                                        int shift, int bits, int64_t num_tiles,
                                                        int64_t* __restrict__ hist) {
  __shared__ uint32_t counts[1 << kMaxDigitBits];
  const int buckets = 1 << bits;
  for (int b = threadIdx.x; b < buckets; b += 64) counts[b] = 0;
  __syncthreads();
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
  for (int c = 0; c < kSortItems; ++c) {
    const int64_t i = base + (int64_t)c * 64 + threadIdx.x;
    if (i < n) atomicAdd(&counts[(uint32_t)(keys[i] >> shift) & (uint32_t)(buckets - 1)], 1u);
  }
  __syncthreads();
  for (int b = threadIdx.x; b < buckets; b += 64)
    hist[(int64_t)b * num_tiles + blockIdx.x] = (int64_t)counts[b];
}

__global__ __launch_bounds__(64) void radix_scatter_kernel(const uint64_t* __restrict__ keys,
                                                           const uint32_t* __restrict__ vals,
                                                           uint64_t* __restrict__ keys_out,
                                                           uint32_t* __restrict__ vals_out, int64_t n,
                                                           int shift, int bits, int64_t num_tiles,
                                                           const int64_t* __restrict__ hist_scanned) {
  __shared__ int64_t cursor[1 << kMaxDigitBits];
  const int buckets = 1 << bits;
  for (int b = threadIdx.x; b < buckets; b += 64)
    cursor[b] = hist_scanned[(int64_t)b * num_tiles + blockIdx.x];
  __syncthreads();
  const int lane = threadIdx.x;
  const uint64_t below = (1ull << lane) - 1ull;
  const int64_t base = (int64_t)blockIdx.x * kSortTile;
  for (int c = 0; c < kSortItems; ++c) {
    const int64_t i = base + (int64_t)c * 64 + lane;
    const bool valid = i < n;
    uint64_t key = 0;
    uint32_t val = 0;
    if (valid) { key = keys[i]; val = vals[i]; }
    const uint32_t digit = (uint32_t)(key >> shift) & (uint32_t)(buckets - 1);
    uint64_t peers = __ballot(valid);
    for (int b = 0; b < bits; ++b) {
      const bool one = (digit >> b) & 1u;
      const uint64_t vote = __ballot(valid && one);
      peers &= one ? vote : ~vote;
    }
    int64_t dest = 0;
    if (valid) dest = cursor[digit] + (int64_t)__popcll(peers & below);
    __syncthreads();
    if (valid && (peers & below) == 0) cursor[digit] += (int64_t)__popcll(peers);
    __syncthreads();
    if (valid) { keys_out[dest] = key; vals_out[dest] = val; }
  }
}

static int64_t sort_tiles(int64_t n) { return ceil_div(n, kSortTile); }

size_t radix_sort_scratch_bytes(int64_t n) {
  const size_t hist = (size_t)sort_tiles(n) << kMaxDigitBits;
  return align_up(hist * 8) + align_up(scan_scratch_elems((int64_t)hist) * 8);
}

int32_t radix_sort_u64_u32(uint64_t* keys, uint32_t* vals, uint64_t* keys_alt, uint32_t* vals_alt,
                           int64_t n, int lo_a, int nbits_a, int lo_b, int nbits_b, void* scratch,
                           hipStream_t stream) {
  if (n <= 0) return GS_OK;
  const int64_t tiles = sort_tiles(n);
  Carver cv(scratch);
  int64_t* hist = cv.take<int64_t>((size_t)tiles << kMaxDigitBits);
  int64_t* scan_scratch = cv.take<int64_t>(scan_scratch_elems(tiles << kMaxDigitBits));
  uint64_t* k_in = keys; uint32_t* v_in = vals;
  uint64_t* k_out = keys_alt; uint32_t* v_out = vals_alt;
  const int lo[2] = {lo_a, lo_b};
  const int nb[2] = {nbits_a, nbits_b};
  for (int f = 0; f < 2; ++f) {
    if (nb[f] <= 0) continue;
    const int passes = (nb[f] + kMaxDigitBits - 1) / kMaxDigitBits;
    const int width = (nb[f] + passes - 1) / passes;
    for (int p = 0; p < passes; ++p) {
      const int shift = lo[f] + p * width;
      const int bits = (p == passes - 1) ? (nb[f] - p * width) : width;
      radix_hist_kernel<<<dim3((unsigned)tiles), 64, 0, stream>>>(k_in, n, shift, bits, tiles, hist);
      GS_LAUNCH_CHECK();
      int32_t rc = exclusive_scan_i64(hist, tiles << bits, scan_scratch, nullptr, stream);
      if (rc != GS_OK) return rc;
      radix_scatter_kernel<<<dim3((unsigned)tiles), 64, 0, stream>>>(k_in, v_in, k_out, v_out, n, shift,
                                                                     bits, tiles, hist);
      GS_LAUNCH_CHECK();
      uint64_t* tk = k_in; k_in = k_out; k_out = tk;
      uint32_t* tv = v_in; v_in = v_out; v_out = tv;
    }
  }
  if (k_in != keys) {
    GS_HIP_TRY(hipMemcpyAsync(keys, k_in, (size_t)n * 8, hipMemcpyDeviceToDevice, stream));
    GS_HIP_TRY(hipMemcpyAsync(vals, v_in, (size_t)n * 4, hipMemcpyDeviceToDevice, stream));
  }
  return GS_OK;
}

}  // namespace gs
