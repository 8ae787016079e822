// Internal helpers shared by the HIP translation units of libdagattn (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "dagattn.h"

#define DAG_HIP_CHECK(expr)                    \
  do {                                         \
    hipError_t e__ = (expr);                   \
    if (e__ != hipSuccess) return DAG_ERR_HIP; \
  } while (0)

#define DAG_LAUNCH_CHECK()                             \
  do {                                                 \
    if (hipGetLastError() != hipSuccess) return DAG_ERR_HIP; \
  } while (0)

static inline bool dag_aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
static inline int64_t dag_ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
static inline size_t dag_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2;

// fp32 -> bf16 bits, round to nearest even (NaN not expected on these paths but kept quiet).
__device__ __forceinline__ uint32_t dag_f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
  u += 0x7fffu + ((u >> 16) & 1u);
  return u >> 16;
}
// Two fp32 -> packed bf16 pair (lo in bits 0..15) with the hardware conversion (round to nearest
// even, one v_cvt_pk_bf16_f32).
__device__ __forceinline__ uint32_t dag_pack_bf2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) float dag_f32x2;
  typedef __attribute__((ext_vector_type(2))) __bf16 dag_bf16x2;
  const dag_f32x2 f = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, dag_bf16x2));
}
__device__ __forceinline__ float dag_bf_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float dag_bf_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// Largest sequence index b with start[b] <= x, for a non-decreasing array start[0..n] (start[0] = 0).
template <typename T>
__device__ __forceinline__ int dag_find_segment(const T* start, int n, T x) {
  int lo = 0, hi = n;  // invariant: start[lo] <= x < start[hi] (conceptually start[n] > x)
  while (hi - lo > 1) {
    int mid = (lo + hi) >> 1;
    if (start[mid] <= x) lo = mid; else hi = mid;
  }
  return lo;
}
