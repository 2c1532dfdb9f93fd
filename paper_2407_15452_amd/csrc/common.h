// Shared host/device helpers of libgs (gfx950 only).
#pragma once

#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/gs.h"

namespace gs {

// ---- host side -------------------------------------------------------------
void set_last_hip_error(hipError_t e);

#define GS_HIP_TRY(expr)                              \
  do {                                                \
    hipError_t e_ = (expr);                           \
    if (e_ != hipSuccess) {                           \
      ::gs::set_last_hip_error(e_);                   \
      return GS_EHIP;                                 \
    }                                                 \
  } while (0)

// Call after a kernel launch: picks up launch-configuration errors.
#define GS_LAUNCH_CHECK() GS_HIP_TRY(hipGetLastError())

inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }
inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Carves 256-byte aligned pieces out of a caller workspace (or just sizes it).
struct Carver {
  char* base;
  size_t used = 0;
  explicit Carver(void* ws) : base(static_cast<char*>(ws)) {}
  template <typename T>
  T* take(size_t count) {
    T* p = base ? reinterpret_cast<T*>(base + used) : nullptr;
    used += align_up(count * sizeof(T));
    return p;
  }
};

// Exclusive prefix sum of n int64 values, in place.  `scratch` must hold
// scan_scratch_elems(n) int64 values.  total_out (device, may be null)
// receives the sum of all n inputs.
size_t scan_scratch_elems(int64_t n);
int32_t exclusive_scan_i64(int64_t* data, int64_t n, int64_t* scratch, int64_t* total_out,
                           hipStream_t stream);

// Stable least-significant-digit radix sort of (key, payload) records on the
// key bits [lo_a, lo_a + nbits_a) then [lo_b, lo_b + nbits_b).  The result is
// left in (keys, vals); (keys_alt, vals_alt) are scratch of the same size.
size_t radix_sort_scratch_bytes(int64_t n);
int32_t radix_sort_u64_u32(uint64_t* keys, uint32_t* vals, uint64_t* keys_alt, uint32_t* vals_alt,
                           int64_t n, int lo_a, int nbits_a, int lo_b, int nbits_b,
                           void* scratch, hipStream_t stream);

// ---- device side -----------------------------------------------------------
#if defined(__HIPCC__)

struct Block4 { uint32_t x0, x1, x2, x3; };

// Philox4x32-10 (Salmon et al., SC'11).
__device__ __forceinline__ Block4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                                uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    // one 32 x 32 -> 64 bit multiply per product (both halves from one instruction)
    const uint64_t pa = (uint64_t)0xD2511F53u * (uint64_t)c0;
    const uint64_t pb = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
    const uint32_t hi_a = (uint32_t)(pa >> 32), lo_a = (uint32_t)pa;
    const uint32_t hi_b = (uint32_t)(pb >> 32), lo_b = (uint32_t)pb;
    c0 = hi_b ^ c1 ^ k0;
    c1 = lo_b;
    c2 = hi_a ^ c3 ^ k1;
    c3 = lo_a;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return Block4{c0, c1, c2, c3};
}

__device__ __forceinline__ Block4 philox_at(uint64_t seed, uint64_t index, uint32_t c2, uint32_t c3) {
  return philox4x32_10((uint32_t)index, (uint32_t)(index >> 32), c2, c3, (uint32_t)seed,
                       (uint32_t)(seed >> 32));
}

__device__ __forceinline__ uint64_t slot_of(const Block4& b, uint64_t n) {
  return __umul64hi(((uint64_t)b.x0 << 32) | (uint64_t)b.x1, n);
}

__device__ __forceinline__ float unit_float(uint32_t x) { return (float)(x >> 8) * 0x1p-24f; }

// One draw from a single alias table of n entries with random block b: words 0,1
// choose the slot, word 2 decides between the slot and its alias.  All three
// table pointers null: uniform.  `packed` (prob bits, alias) is read when present.
__device__ __forceinline__ int64_t table_draw(const float* __restrict__ prob,
                                              const int32_t* __restrict__ alias,
                                              const uint2* __restrict__ packed, uint64_t n,
                                              const Block4& b) {
  int64_t s = (int64_t)slot_of(b, n);
  if (packed != nullptr) {
    const uint2 e = packed[s];                      // one 8-byte load
    if (!(unit_float(b.x2) < __uint_as_float(e.x))) s = (int64_t)(int32_t)e.y;
  } else if (prob != nullptr) {
    if (!(unit_float(b.x2) < prob[s])) s = (int64_t)alias[s];
  }
  return s;
}

// 16-bit storage formats of the embedding tables.  lo / hi widen the two halves of a
// 32-bit word exactly; round() gives the 16 bits nearest to an fp32 value (ties to even).
struct bf16_t {
  uint16_t bits;
  static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
  static __device__ __forceinline__ uint32_t round(float f) {      // finite inputs
    const uint32_t b = __float_as_uint(f);
    return (b + 0x7fffu + ((b >> 16) & 1u)) >> 16;
  }
};
struct f16_t {                                                      // IEEE binary16
  uint16_t bits;
  static __device__ __forceinline__ float lo(uint32_t w) {
    return __half2float(__ushort_as_half((unsigned short)(w & 0xffffu)));
  }
  static __device__ __forceinline__ float hi(uint32_t w) {
    return __half2float(__ushort_as_half((unsigned short)(w >> 16)));
  }
  static __device__ __forceinline__ uint32_t round(float f) {
    // The value is an fp32 result first and becomes 16 bits by a second rounding.  Left to
    // itself the compiler may merge the producing multiply / add into one mixed-precision
    // instruction that rounds the exact result once, which gives other bits on ties.
    asm("" : "+v"(f));
    return (uint32_t)__half_as_ushort(__float2half_rn(f));
  }
};
template <typename T>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
  return T::round(lo) | (T::round(hi) << 16);
}

// ---- skip-gram pair numbering inside one walk (Sec. 2.2; order: position, then offset) ----
// f(x) = sum_{m=0}^{x-1} min(m, W).  A walk prefix of `len` nodes has
// C(a) = f(a) + f(len) - f(len - a) pairs before position a, 2 f(len) in all.
__device__ __forceinline__ int64_t window_prefix(int64_t x, int64_t w) {
  return (x <= w + 1) ? x * (x - 1) / 2 : w * (w + 1) / 2 + (x - w - 1) * w;
}
__device__ __forceinline__ int64_t pairs_before(int64_t a, int64_t len, int64_t w) {
  return window_prefix(a, w) + window_prefix(len, w) - window_prefix(len - a, w);
}

// length of the non-negative prefix of a row (-1 only ever forms a suffix)
__device__ __forceinline__ int32_t valid_prefix(const int32_t* row, int32_t walk_len) {
  int32_t lo = 0, hi = walk_len;
  while (lo < hi) {
    const int32_t mid = (lo + hi) >> 1;
    if (row[mid] >= 0) lo = mid + 1; else hi = mid;
  }
  return lo;
}

// pair number q (0-based) of a walk prefix of `len` nodes: centre position a, context position
__device__ __forceinline__ void pair_positions(int64_t q, int64_t len, int64_t window, int64_t& a,
                                               int64_t& other) {
  int64_t alo = 0, ahi = len - 1;                 // last a with pairs_before(a) <= q
  while (alo < ahi) {
    const int64_t mid = (alo + ahi + 1) >> 1;
    if (pairs_before(mid, len, window) <= q) alo = mid; else ahi = mid - 1;
  }
  a = alo;
  other = max((int64_t)0, a - window) + (q - pairs_before(a, len, window));
  if (other >= a) ++other;
}

template <typename OffT>
__device__ __forceinline__ int64_t load_off(const void* offsets, int64_t i) {
  return (int64_t) static_cast<const OffT*>(offsets)[i];
}

#endif  // __HIPCC__

}  // namespace gs
