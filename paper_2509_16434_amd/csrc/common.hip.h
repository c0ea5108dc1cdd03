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
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));  // one v_cvt_pk_bf16_f32
}

// 16-byte store of data that is not read again soon (an activation written for a later kernel): non-temporal,
// so that it does not displace the inputs in the caches
__device__ __forceinline__ void store_stream16(bf16_t* p, const uint4& v) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(p));
}

// Division of n < 2^31 by a launch constant d >= 1 without a divide: with 2^sh < d <= 2^(sh+1)
// and mul = floor(2^(32+sh) / d) + 1, floor(n / d) = (n * mul) >> (32 + sh) exactly (the error
// term n * (mul*d - 2^(32+sh)) stays below 2^(32+sh)).  d == 0 marks "not prepared".
struct FastDiv {
  uint32_t mul = 0, sh = 0, d = 0;
  __device__ __forceinline__ uint32_t div(uint32_t n) const { return d == 1u ? n : (__umulhi(n, mul) >> sh); }
};
inline FastDiv make_fastdiv(int32_t d) {
  FastDiv f;
  f.d = (uint32_t)d;
  if (d > 1) {
    uint32_t sh = 0;
    while ((2u << sh) < (uint32_t)d) ++sh;
    f.sh = sh;
    f.mul = (uint32_t)((((uint64_t)1 << (32 + sh)) / (uint32_t)d) + 1);
  }
  return f;
}

// Blocks are dealt to the eight XCDs (each with its own L2) round-robin: block b runs on XCD b % 8.  xcd_block
// renumbers the blocks so that those of one XCD get consecutive numbers; the tile kernels deal their tiles by
// that number, so that neighbouring bands of an image, which share input rows, are worked on at the same time
// by CUs behind the same L2.  A permutation when nb is a multiple of 8, else the identity.
__device__ __forceinline__ int xcd_block(int b, int nb) { return (nb & 7) == 0 ? (b & 7) * (nb >> 3) + (b >> 3) : b; }

// Address of image `img` (= sample*V + view) inside a tensor whose samples may be gathered
// through an index list and whose views sit at a fixed stride inside a sample row.
struct ImgAddr {
  const bf16_t* base;
  const int32_t* idx;  // optional sample gather (NULL = identity)
  int64_t stride_b;    // elements between consecutive samples
  int64_t stride_v;    // elements between views of one sample
  int32_t V;
  FastDiv dv;          // optional: set by prepare()
  void prepare() { dv = make_fastdiv(V); }
  __device__ __forceinline__ const bf16_t* ptr(int img) const {
    int b = img, v = 0;
    if (V != 1) { b = (dv.d == (uint32_t)V) ? (int)dv.div((uint32_t)img) : img / V; v = img - b * V; }
    int64_t s = idx ? (int64_t)idx[b] : (int64_t)b;
    return base + s * stride_b + (int64_t)v * stride_v;
  }
  // The same for a wave-uniform image number.  The gather index is read through the constant address
  // space, hence with a scalar load: a vector load here would make the caller wait for every
  // vector-memory operation it has in flight (LDS-writing band loads included) before it can form
  // the address.  The index list is never written by a kernel that reads it this way.
  __device__ __forceinline__ const bf16_t* ptr_uniform(int img) const {
    int b = img, v = 0;
    if (V != 1) { b = (dv.d == (uint32_t)V) ? (int)dv.div((uint32_t)img) : img / V; v = img - b * V; }
    b = __builtin_amdgcn_readfirstlane(b);
    typedef const __attribute__((address_space(4))) int32_t* cidx_t;
    int64_t s = idx ? (int64_t)reinterpret_cast<cidx_t>(reinterpret_cast<uintptr_t>(idx))[b] : (int64_t)b;
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
