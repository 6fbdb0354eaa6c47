// Small device helpers shared by the kernels: bf16 <-> fp32 conversion and typed loads/stores.
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>

namespace dcp {

typedef uint16_t bf16_t;  // raw bits

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// two floats to two bf16 in one 32-bit word (lo in the low half), rounded to nearest even by the hardware conversion
// (one instruction for the pair; the software routine above costs about six per value)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  typedef __bf16 hb2 __attribute__((ext_vector_type(2)));
  typedef float f2 __attribute__((ext_vector_type(2)));
  const f2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, hb2));
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Visibility of packed key index j under one table row for the query with packed index i.
// lo/hi are the row's two ranges already loaded (RANGES), c0/c1 the KV block's token range.
__device__ __forceinline__ bool key_visible(int kind, int i, int j, int4 r) {
  if (kind == 0) return true;
  if (kind == 1) return j <= i;
  return (j >= r.x && j < r.y) || (j >= r.z && j < r.w);
}

}  // namespace dcp
