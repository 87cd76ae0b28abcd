// Storage types and conversions used by the device code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gs {

typedef uint16_t bf16_t;   // bfloat16 bit pattern

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float floatx4_t;

__device__ __forceinline__ float bf16_to_float(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

typedef __bf16 bf16x2_native_t __attribute__((ext_vector_type(2)));
typedef float float2_native_t __attribute__((ext_vector_type(2)));

// two floats -> two bfloat16 in one 32-bit word (low half first); round to nearest, ties to even
// (the hardware packed conversion of gfx950)
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  const float2_native_t v = {lo, hi};
  const bf16x2_native_t b = __builtin_convertvector(v, bf16x2_native_t);
  return *reinterpret_cast<const uint32_t*>(&b);
}

__device__ __forceinline__ bf16_t float_to_bf16(float f) { return (bf16_t)(pack_bf16x2(f, 0.f) & 0xffffu); }

template <typename T> struct Storage;
template <> struct Storage<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Storage<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_float(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = float_to_bf16(v); }
};

}  // namespace gs
