// gs_sgns_step: one SGNS training iteration (GraphScale Sec. 3.2: fetch the
// rows the batch names, loss and sparse gradient on them, write them back, with
// the barrier of "Synchronization": all reads see the pre-iteration tables).
//
// The batch-synchronous rule is kept by splitting the iteration at kernel
// boundaries:
//   forward   read-only on both tables: logits, g = dLoss/dx, loss, and the
//             centre-row gradients staged per run of equal centres;
//   scatter   w_out[row] += -lr * g * u   (atomic, reads the unmodified w_in);
//   apply     w_in[centre] += -lr * staged gradient (atomic);
//   finish    deterministic sum of the per-block loss partials.
// A row is handled by 16 lanes holding float4 pieces (256 contiguous bytes per
// load instruction); a wave works on four rows at once and a dot product is a
// 16-lane DPP reduction.  No matrix cores: 0.3 flop per byte moved.
#include "common.h"

namespace gs {

constexpr int kSgnsThreads = 256;
constexpr int kGroupLanes = 16;
constexpr int kGroupsPerBlock = kSgnsThreads / kGroupLanes;
constexpr int kChunkPairs = 16;   // consecutive pairs per 16-lane group
constexpr int kRowBatch = 3;      // rows whose loads are issued together

struct SgnsArgs {
  float* w_in;
  float* w_out;
  const int32_t* centers;
  const int32_t* contexts;
  const int32_t* negs;
  int64_t num_pairs;
  int32_t k;
  int32_t dim;
  float lr;
  float* g;                 // [num_pairs][k+1]
  unsigned long long* slot_counter;
  int32_t* stage_center;    // [<= num_pairs]
  float* stage_delta;       // [<= num_pairs][dim]
  double* loss_partials;    // [forward blocks]
  int64_t forward_blocks;
  double* loss_out;
};

// sum over the 16 lanes of a DPP row; every lane gets the total
__device__ __forceinline__ float row_sum16(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // quad_perm [1,0,3,2]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // quad_perm [2,3,0,1]
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // row_half_mirror
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x140, 0xF, 0xF, true));  // row_mirror
  return x;
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

template <int VPL>
__device__ __forceinline__ float dot_partial(const float4 (&a)[VPL], const float4 (&b)[VPL]) {
  float s = 0.f;
#pragma unroll
  for (int v = 0; v < VPL; ++v)
    s += a[v].x * b[v].x + a[v].y * b[v].y + a[v].z * b[v].z + a[v].w * b[v].w;
  return s;
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }
__device__ __forceinline__ float softplusf_(float z) {
  return fmaxf(z, 0.0f) + log1pf(expf(-fabsf(z)));
}

template <int VPL>
__device__ __forceinline__ void stage_flush(const SgnsArgs& a, int32_t center, int l16,
                                            const float4 (&du)[VPL]) {
  unsigned long long slot = 0;
  if (l16 == 0) slot = atomicAdd(a.slot_counter, 1ull);
  slot = __shfl(slot, 0, kGroupLanes);
  if (l16 == 0) a.stage_center[slot] = center;
  float4* out = reinterpret_cast<float4*>(a.stage_delta + (int64_t)slot * a.dim);
  const int dim4 = a.dim >> 2;
#pragma unroll
  for (int v = 0; v < VPL; ++v) {
    const int q = v * kGroupLanes + l16;
    if (q < dim4) out[q] = du[v];
  }
}

template <int VPL>
__global__ __launch_bounds__(kSgnsThreads) void sgns_forward_kernel(SgnsArgs a) {
  __shared__ float loss_s[kGroupsPerBlock];
  const int l16 = threadIdx.x & (kGroupLanes - 1);
  const int group_in_block = threadIdx.x / kGroupLanes;
  const int64_t group = (int64_t)blockIdx.x * kGroupsPerBlock + group_in_block;
  const int64_t first = group * kChunkPairs;
  const int64_t last = min(first + kChunkPairs, a.num_pairs);
  const int K = a.k;

  float4 u[VPL], du[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) { u[v] = make_float4(0.f, 0.f, 0.f, 0.f); du[v] = u[v]; }
  int32_t cur_c = -1;
  float loss = 0.f;

  for (int64_t i = first; i < last; ++i) {
    const int32_t c = a.centers[i];
    if (c != cur_c) {
      if (cur_c >= 0) stage_flush<VPL>(a, cur_c, l16, du);
      load_row<VPL>(a.w_in, c, a.dim, l16, u);
#pragma unroll
      for (int v = 0; v < VPL; ++v) du[v] = make_float4(0.f, 0.f, 0.f, 0.f);
      cur_c = c;
    }
    for (int j0 = 0; j0 <= K; j0 += kRowBatch) {
      float4 vv[kRowBatch][VPL];
#pragma unroll
      for (int b = 0; b < kRowBatch; ++b) {
        const int j = j0 + b;
        if (j <= K) {
          const int32_t row = (j == 0) ? a.contexts[i] : a.negs[i * (int64_t)K + (j - 1)];
          load_row<VPL>(a.w_out, row, a.dim, l16, vv[b]);
        }
      }
#pragma unroll
      for (int b = 0; b < kRowBatch; ++b) {
        const int j = j0 + b;
        if (j <= K) {
          const float x = row_sum16(dot_partial<VPL>(u, vv[b]));
          float gj;
          if (j == 0) { gj = sigmoidf_(x) - 1.0f; loss += softplusf_(-x); }
          else        { gj = sigmoidf_(x);        loss += softplusf_(x); }
#pragma unroll
          for (int v = 0; v < VPL; ++v) {
            du[v].x += gj * vv[b][v].x; du[v].y += gj * vv[b][v].y;
            du[v].z += gj * vv[b][v].z; du[v].w += gj * vv[b][v].w;
          }
          if (l16 == 0) a.g[i * (int64_t)(K + 1) + j] = gj;
        }
      }
    }
  }
  if (cur_c >= 0) stage_flush<VPL>(a, cur_c, l16, du);

  if (l16 == 0) loss_s[group_in_block] = loss;
  __syncthreads();
  if (threadIdx.x == 0) {
    double s = 0.0;
#pragma unroll
    for (int gidx = 0; gidx < kGroupsPerBlock; ++gidx) s += (double)loss_s[gidx];
    a.loss_partials[blockIdx.x] = s;
  }
}

template <int VPL>
__global__ __launch_bounds__(kSgnsThreads) void sgns_scatter_kernel(SgnsArgs a) {
  const int l16 = threadIdx.x & (kGroupLanes - 1);
  const int64_t group = ((int64_t)blockIdx.x * kSgnsThreads + threadIdx.x) / kGroupLanes;
  const int64_t first = group * kChunkPairs;
  const int64_t last = min(first + kChunkPairs, a.num_pairs);
  const int K = a.k;
  const int dim4 = a.dim >> 2;
  float4 u[VPL];
#pragma unroll
  for (int v = 0; v < VPL; ++v) u[v] = make_float4(0.f, 0.f, 0.f, 0.f);
  int32_t cur_c = -1;
  for (int64_t i = first; i < last; ++i) {
    const int32_t c = a.centers[i];
    if (c != cur_c) { load_row<VPL>(a.w_in, c, a.dim, l16, u); cur_c = c; }
    for (int j = 0; j <= K; ++j) {
      const int32_t row = (j == 0) ? a.contexts[i] : a.negs[i * (int64_t)K + (j - 1)];
      const float coef = -a.lr * a.g[i * (int64_t)(K + 1) + j];
      float* dst = a.w_out + row * (int64_t)a.dim;
#pragma unroll
      for (int v = 0; v < VPL; ++v) {
        const int q = v * kGroupLanes + l16;
        if (q < dim4) {
          unsafeAtomicAdd(dst + 4 * q + 0, coef * u[v].x);
          unsafeAtomicAdd(dst + 4 * q + 1, coef * u[v].y);
          unsafeAtomicAdd(dst + 4 * q + 2, coef * u[v].z);
          unsafeAtomicAdd(dst + 4 * q + 3, coef * u[v].w);
        }
      }
    }
  }
}

template <int VPL>
__global__ __launch_bounds__(kSgnsThreads) void sgns_apply_kernel(SgnsArgs a) {
  const int l16 = threadIdx.x & (kGroupLanes - 1);
  const int64_t group = ((int64_t)blockIdx.x * kSgnsThreads + threadIdx.x) / kGroupLanes;
  const int64_t stride = (int64_t)gridDim.x * kGroupsPerBlock;
  const int64_t slots = (int64_t)*a.slot_counter;
  const int dim4 = a.dim >> 2;
  for (int64_t s = group; s < slots; s += stride) {
    const int32_t c = a.stage_center[s];
    const float4* src = reinterpret_cast<const float4*>(a.stage_delta + s * (int64_t)a.dim);
    float* dst = a.w_in + c * (int64_t)a.dim;
#pragma unroll
    for (int v = 0; v < VPL; ++v) {
      const int q = v * kGroupLanes + l16;
      if (q < dim4) {
        const float4 d = src[q];
        unsafeAtomicAdd(dst + 4 * q + 0, -a.lr * d.x);
        unsafeAtomicAdd(dst + 4 * q + 1, -a.lr * d.y);
        unsafeAtomicAdd(dst + 4 * q + 2, -a.lr * d.z);
        unsafeAtomicAdd(dst + 4 * q + 3, -a.lr * d.w);
      }
    }
  }
}

__global__ void sgns_init_kernel(unsigned long long* slot_counter) { *slot_counter = 0ull; }

__global__ __launch_bounds__(256) void sgns_finish_kernel(const double* __restrict__ partials,
                                                          int64_t count, double* __restrict__ out) {
  __shared__ double s[256];
  double acc = 0.0;
  for (int64_t i = threadIdx.x; i < count; i += 256) acc += partials[i];
  s[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) s[threadIdx.x] += s[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) *out = s[0];
}

static int64_t forward_blocks_for(int64_t num_pairs) {
  return ceil_div(ceil_div(num_pairs, kChunkPairs), kGroupsPerBlock);
}

struct SgnsPlan {
  unsigned long long* slot_counter;
  double* loss_partials;
  float* g;
  int32_t* stage_center;
  float* stage_delta;
  size_t bytes;
};

static SgnsPlan plan_sgns(void* ws, int64_t num_pairs, int32_t k, int32_t dim) {
  Carver cv(ws);
  SgnsPlan p;
  const size_t b = (size_t)(num_pairs > 0 ? num_pairs : 1);
  p.slot_counter = cv.take<unsigned long long>(1);
  p.loss_partials = cv.take<double>((size_t)forward_blocks_for((int64_t)b));
  p.g = cv.take<float>(b * (size_t)(k + 1));
  p.stage_center = cv.take<int32_t>(b);
  p.stage_delta = cv.take<float>(b * (size_t)dim);
  p.bytes = cv.used;
  return p;
}

template <int VPL>
static int32_t launch_sgns(const SgnsArgs& a, hipStream_t stream) {
  const unsigned blocks = (unsigned)a.forward_blocks;
  sgns_init_kernel<<<1, 1, 0, stream>>>(a.slot_counter);
  GS_LAUNCH_CHECK();
  sgns_forward_kernel<VPL><<<blocks, kSgnsThreads, 0, stream>>>(a);
  GS_LAUNCH_CHECK();
  sgns_scatter_kernel<VPL><<<blocks, kSgnsThreads, 0, stream>>>(a);
  GS_LAUNCH_CHECK();
  const unsigned apply_blocks = blocks < 2048u ? blocks : 2048u;
  sgns_apply_kernel<VPL><<<apply_blocks, kSgnsThreads, 0, stream>>>(a);
  GS_LAUNCH_CHECK();
  sgns_finish_kernel<<<1, 256, 0, stream>>>(a.loss_partials, a.forward_blocks, a.loss_out);
  GS_LAUNCH_CHECK();
  return GS_OK;
}

__global__ void zero_double_kernel(double* p) { *p = 0.0; }

}  // namespace gs

using namespace gs;

extern "C" size_t gs_sgns_step_workspace_bytes(int64_t num_pairs, int32_t k, int32_t dim,
                                               int32_t dtype) {
  (void)dtype;
  if (num_pairs < 0 || k < 0 || dim < 1) return 0;
  return plan_sgns(nullptr, num_pairs, k, dim).bytes;
}

extern "C" int32_t gs_sgns_step(void* w_in, void* w_out, int64_t num_nodes, int32_t dim,
                                int32_t dtype, const int32_t* centers, const int32_t* contexts,
                                const int32_t* negs, int64_t num_pairs, int32_t k, float lr,
                                double* loss_sum_out, void* ws, size_t ws_bytes, void* stream_) {
  hipStream_t stream = (hipStream_t)stream_;
  if (!w_in || !w_out || num_nodes < 1 || num_nodes > (int64_t)INT32_MAX) return GS_EINVAL;
  if (dim < 4 || dim > 1024 || (dim & 3) != 0) return GS_EINVAL;
  if (dtype != GS_F32) return GS_EINVAL;   // bf16 tables: not built yet
  if (num_pairs < 0 || k < 0 || !loss_sum_out) return GS_EINVAL;
  if (num_pairs > 0 && (!centers || !contexts || (k > 0 && !negs))) return GS_EINVAL;
  if (!aligned(w_in, 16) || !aligned(w_out, 16)) return GS_EINVAL;
  if (!ws || !aligned(ws, 256)) return GS_EINVAL;
  SgnsPlan p = plan_sgns(ws, num_pairs, k, dim);
  if (ws_bytes < p.bytes) return GS_EWORKSPACE;
  if (num_pairs == 0) {
    zero_double_kernel<<<1, 1, 0, stream>>>(loss_sum_out);
    GS_LAUNCH_CHECK();
    return GS_OK;
  }
  SgnsArgs a;
  a.w_in = (float*)w_in;
  a.w_out = (float*)w_out;
  a.centers = centers;
  a.contexts = contexts;
  a.negs = negs;
  a.num_pairs = num_pairs;
  a.k = k;
  a.dim = dim;
  a.lr = lr;
  a.g = p.g;
  a.slot_counter = p.slot_counter;
  a.stage_center = p.stage_center;
  a.stage_delta = p.stage_delta;
  a.loss_partials = p.loss_partials;
  a.forward_blocks = forward_blocks_for(num_pairs);
  a.loss_out = loss_sum_out;
  const int vpl = (dim + 63) / 64;
  if (vpl <= 1) return launch_sgns<1>(a, stream);
  if (vpl <= 2) return launch_sgns<2>(a, stream);
  if (vpl <= 4) return launch_sgns<4>(a, stream);
  if (vpl <= 8) return launch_sgns<8>(a, stream);
  return launch_sgns<16>(a, stream);
}
