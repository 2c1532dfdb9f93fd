// gs_csr_build: edge list -> CSR on the device (GraphScale Sec. 3.1: the
// topology a trainer keeps).  Records (src << 32 | dst, input index) are sorted
// stably, duplicates are flagged, and the survivors are compacted.
#include "common.h"

namespace gs {

constexpr uint64_t kDroppedKey = ~0ull;

__global__ void csr_keygen_kernel(const int32_t* __restrict__ src, const int32_t* __restrict__ dst,
                                  int64_t cap, int64_t num_nodes, uint32_t flags,
                                  uint64_t* __restrict__ keys, uint32_t* __restrict__ vals) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= cap) return;
  const bool sym = flags & GS_SYMMETRIZE;
  const int64_t i = sym ? (e >> 1) : e;
  int32_t s = src[i], d = dst[i];
  if (sym && (e & 1)) { int32_t t = s; s = d; d = t; }
  const bool ok = s >= 0 && d >= 0 && s < num_nodes && d < num_nodes &&
                  !((flags & GS_DROP_SELF_LOOPS) && s == d);
  keys[e] = ok ? (((uint64_t)(uint32_t)s << 32) | (uint64_t)(uint32_t)d) : kDroppedKey;
  vals[e] = (uint32_t)i;
}

__device__ __forceinline__ bool csr_keeps(const uint64_t* keys, int64_t e, bool dedupe) {
  const uint64_t k = keys[e];
  if (k == kDroppedKey) return false;
  return !(dedupe && e > 0 && keys[e - 1] == k);
}

__global__ void csr_flag_kernel(const uint64_t* __restrict__ keys, int64_t cap, uint32_t flags,
                                int64_t* __restrict__ pos) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e < cap) pos[e] = csr_keeps(keys, e, flags & GS_DEDUPE) ? 1 : 0;
}

__global__ void csr_compact_kernel(const uint64_t* __restrict__ keys, const uint32_t* __restrict__ vals,
                                   const int64_t* __restrict__ pos, int64_t cap, uint32_t flags,
                                   const float* __restrict__ w, int32_t* __restrict__ nbrs_out,
                                   float* __restrict__ w_out, int32_t* __restrict__ row_of) {
  const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (e >= cap || !csr_keeps(keys, e, flags & GS_DEDUPE)) return;
  const int64_t p = pos[e];
  const uint64_t k = keys[e];
  nbrs_out[p] = (int32_t)(uint32_t)k;
  row_of[p] = (int32_t)(uint32_t)(k >> 32);
  if (w != nullptr) w_out[p] = w[vals[e]];
}

// offsets[v] = number of kept entries whose row is < v  (lower bound in row_of)
template <typename OffT>
__global__ void csr_offsets_kernel(const int32_t* __restrict__ row_of,
                                   const int64_t* __restrict__ num_entries, int64_t num_nodes,
                                   OffT* __restrict__ offsets) {
  const int64_t v = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (v > num_nodes) return;
  int64_t lo = 0, hi = *num_entries;
  while (lo < hi) {
    const int64_t mid = lo + ((hi - lo) >> 1);
    if ((int64_t)row_of[mid] < v) lo = mid + 1; else hi = mid;
  }
  offsets[v] = (OffT)lo;
}

static int bits_for(int64_t n) {  // bits needed for ids in [0, n)
  int b = 1;
  while (b < 32 && ((int64_t)1 << b) < n) ++b;
  return b;
}

struct CsrPlan {
  uint64_t *keys, *keys_alt;
  uint32_t *vals, *vals_alt;
  int64_t *pos, *scan_scratch;
  int32_t* row_of;
  void* sort_scratch;
  size_t bytes;
};

static CsrPlan plan_csr(void* ws, int64_t cap) {
  Carver cv(ws);
  CsrPlan p;
  const size_t c = (size_t)(cap > 0 ? cap : 1);
  p.keys = cv.take<uint64_t>(c);
  p.keys_alt = cv.take<uint64_t>(c);
  p.vals = cv.take<uint32_t>(c);
  p.vals_alt = cv.take<uint32_t>(c);
  p.pos = cv.take<int64_t>(c);
  p.scan_scratch = cv.take<int64_t>(scan_scratch_elems((int64_t)c));
  p.row_of = cv.take<int32_t>(c);
  p.sort_scratch = cv.take<char>(radix_sort_scratch_bytes((int64_t)c));
  p.bytes = cv.used;
  return p;
}

}  // namespace gs

using namespace gs;

extern "C" size_t gs_csr_build_workspace_bytes(int64_t m, int64_t num_nodes, uint32_t flags) {
  (void)num_nodes;
  if (m < 0) return 0;
  const int64_t cap = (flags & GS_SYMMETRIZE) ? 2 * m : m;
  return plan_csr(nullptr, cap).bytes;
}

extern "C" int32_t gs_csr_build(const int32_t* src, const int32_t* dst, const float* w, int64_t m,
                                int64_t num_nodes, uint32_t flags, int32_t offset_bits,
                                void* offsets_out, int32_t* nbrs_out, float* w_out,
                                int64_t* num_entries_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (m < 0 || num_nodes < 0 || num_nodes > (int64_t)INT32_MAX) return GS_EINVAL;
  if (offset_bits != 32 && offset_bits != 64) return GS_EINVAL;
  if (flags & ~(uint32_t)(GS_SYMMETRIZE | GS_DROP_SELF_LOOPS | GS_DEDUPE)) return GS_EINVAL;
  if (m > 0 && (!src || !dst)) return GS_EINVAL;
  if (!offsets_out || !num_entries_out) return GS_EINVAL;
  if (w != nullptr && w_out == nullptr) return GS_EINVAL;
  if (m > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  const int64_t cap = (flags & GS_SYMMETRIZE) ? 2 * m : m;
  if (offset_bits == 32 && cap > (int64_t)INT32_MAX) return GS_EOVERFLOW;
  if (cap > 0 && !nbrs_out) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  CsrPlan p = plan_csr(ws, cap);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;

  const int threads = 256;
  if (cap > 0) {
    const unsigned blocks = (unsigned)ceil_div(cap, threads);
    csr_keygen_kernel<<<blocks, threads, 0, stream>>>(src, dst, cap, num_nodes, flags, p.keys, p.vals);
    GS_LAUNCH_CHECK();
    const int nb = bits_for(num_nodes);
    // dst field first, then src field with one extra bit so dropped records sort last
    int32_t rc = radix_sort_u64_u32(p.keys, p.vals, p.keys_alt, p.vals_alt, cap, 0, nb, 32, nb + 1,
                                    p.sort_scratch, stream);
    if (rc != GS_OK) return rc;
    csr_flag_kernel<<<blocks, threads, 0, stream>>>(p.keys, cap, flags, p.pos);
    GS_LAUNCH_CHECK();
  }
  int32_t rc = exclusive_scan_i64(p.pos, cap, p.scan_scratch, num_entries_out, stream);
  if (rc != GS_OK) return rc;
  if (cap > 0) {
    const unsigned blocks = (unsigned)ceil_div(cap, threads);
    csr_compact_kernel<<<blocks, threads, 0, stream>>>(p.keys, p.vals, p.pos, cap, flags, w, nbrs_out,
                                                       w_out, p.row_of);
    GS_LAUNCH_CHECK();
  }
  const unsigned oblocks = (unsigned)ceil_div(num_nodes + 1, threads);
  if (offset_bits == 64)
    csr_offsets_kernel<int64_t><<<oblocks, threads, 0, stream>>>(p.row_of, num_entries_out, num_nodes,
                                                                (int64_t*)offsets_out);
  else
    csr_offsets_kernel<int32_t><<<oblocks, threads, 0, stream>>>(p.row_of, num_entries_out, num_nodes,
                                                                (int32_t*)offsets_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}
