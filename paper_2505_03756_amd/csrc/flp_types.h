// Storage-format helpers shared by the kernel translation units (device code only).
#pragma once
#include <hip/hip_runtime.h>

#include <cstdint>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

struct F32 {
  typedef float storage;
  static __device__ __forceinline__ float to_float(float v) { return v; }
  static __device__ __forceinline__ float from_float(float v) { return v; }
};
struct F16 {
  typedef uint16_t storage;
  static __device__ __forceinline__ float to_float(uint16_t v) {
    _Float16 h;
    __builtin_memcpy(&h, &v, 2);
    return (float)h;
  }
  static __device__ __forceinline__ uint16_t from_float(float f) {
    _Float16 h = (_Float16)f;   // round to nearest even
    uint16_t v;
    __builtin_memcpy(&v, &h, 2);
    return v;
  }
};
struct BF16 {
  typedef uint16_t storage;
  static __device__ __forceinline__ float to_float(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
  static __device__ __forceinline__ uint16_t from_float(float f) {
    // nearest even, NaN stays NaN: the hardware conversion of gfx950 (one instruction per two values where the
    // compiler can pair them, against five ALU operations per value by hand)
    const __bf16 b = (__bf16)f;
    uint16_t u;
    __builtin_memcpy(&u, &b, 2);
    return u;
  }
};
