// Shared device-side helpers of the learner kernels (gfx950 / CDNA4, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned short bf16_t;  // raw bfloat16 bits in memory
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;  // one MFMA A/B operand (8 k-values per lane)
typedef __attribute__((ext_vector_type(16))) float f32x16_t;  // one 32x32 MFMA accumulator (16 values per lane)

#define WAVE 64

__device__ __forceinline__ bf16_t f2bf(float f) {
  // round to nearest even (the compiler's fptrunc to bf16)
  __bf16 h = (__bf16)f;
  return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

__device__ __forceinline__ uint32_t pack2bf(float lo, float hi) {
  return (uint32_t)f2bf(lo) | ((uint32_t)f2bf(hi) << 16);
}

// Address of image `img` (= sample*V + view) inside a tensor whose samples may be gathered
// through an index list and whose views sit at a fixed stride inside a sample row.
struct ImgAddr {
  const bf16_t* base;
  const int32_t* idx;  // optional sample gather (NULL = identity)
  int64_t stride_b;    // elements between consecutive samples
  int64_t stride_v;    // elements between views of one sample
  int32_t V;
  __device__ __forceinline__ const bf16_t* ptr(int img) const {
    int b = img / V, v = img - b * V;
    int64_t s = idx ? (int64_t)idx[b] : (int64_t)b;
    return base + s * stride_b + (int64_t)v * stride_v;
  }
};
// Mutable twin for outputs.
struct ImgAddrW {
  bf16_t* base;
  int64_t stride_b, stride_v;
  int32_t V;
  __device__ __forceinline__ bf16_t* ptr(int img) const {
    int b = img / V, v = img - b * V;
    return base + (int64_t)b * stride_b + (int64_t)v * stride_v;
  }
};
