// Plain kernels that show what this GPU reaches: a streaming copy with 16-byte accesses, its read-only and
// store-only halves, the same copy with non-temporal accesses, a register-resident bf16 MFMA loop, and a loop of
// one MFMA followed by K other vector instructions (do the two kinds run side by side on a SIMD?).  Used by
// ppo_diag_peak only; the learner's kernels are priced against the published peaks, these figures sit beside them.
#pragma once
#include "common.hip.h"

enum { PEAK_COPY = 0, PEAK_READ = 1, PEAK_WRITE = 2, PEAK_COPY_NT = 3, PEAK_MFMA = 4, PEAK_MFMA_VALU = 5 };

// Grid-stride over n16 16-byte pieces, four pieces in flight per thread.
template <int MODE>
__global__ __launch_bounds__(256) void k_peak_stream(const uint4* __restrict__ src, uint4* __restrict__ dst, int64_t n16, uint32_t* __restrict__ sink) {
  typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint32_t acc = 0;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    uint4 v[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (MODE == PEAK_WRITE) v[j] = make_uint4((uint32_t)i, j, 0, 0);
      else if (MODE == PEAK_COPY_NT) { const u32x4_t w = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(src + i + j * stride)); v[j] = make_uint4(w.x, w.y, w.z, w.w); }
      else v[j] = src[i + j * stride];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (MODE == PEAK_READ) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
      else if (MODE == PEAK_COPY_NT) { const u32x4_t w = {v[j].x, v[j].y, v[j].z, v[j].w}; __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t*>(dst + i + j * stride)); }
      else dst[i + j * stride] = v[j];
    }
  }
  for (; i < n16; i += stride) {
    if (MODE == PEAK_WRITE) dst[i] = make_uint4((uint32_t)i, 0, 0, 0);
    else if (MODE == PEAK_READ) { const uint4 v = src[i]; acc ^= v.x ^ v.y ^ v.z ^ v.w; }
    else dst[i] = src[i];
  }
  if (MODE == PEAK_READ && acc == 0x9e3779b9u) *sink = acc;  // keeps the loads alive; the buffer holds zeros
}

// Every wave keeps four independent 32x32 accumulators and issues `iters` rounds of four 32x32x16 bf16 MFMAs on
// operands that never leave registers: 4 * 32768 flop per wave per round.
__global__ __launch_bounds__(512) void k_peak_mfma(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8_t a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)(float)((lane + j) & 3); b[j] = (__bf16)(float)((lane * 3 + j) & 1); }
  f32x16_t acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[q][e];
  if (s == -1.f) sink[0] = s;  // never true (all products are >= 0): keeps the loop alive
}

// Do MFMAs and other vector instructions overlap on a SIMD?  Every wave (two per SIMD) issues rounds of eight groups of
// one v_mfma_f32_16x16x32_bf16 (four independent accumulators in turn) followed by K independent v_xor_b32 on K
// registers of their own; nothing depends on anything nearby.  16384 flop per wave per group.  If the two kinds ran
// side by side, the time per group would stay that of the MFMA (16 cycles) up to K = 4.
typedef float f32x4_peak_t __attribute__((ext_vector_type(4)));
template <int K>
__global__ __launch_bounds__(512) void k_peak_mfma_valu(int iters, float* __restrict__ sink) {
  const int lane = threadIdx.x & 63;
  bf16x8_t a, b;
#pragma unroll
  for (int j = 0; j < 8; ++j) { a[j] = (__bf16)(float)((lane + j) & 3); b[j] = (__bf16)(float)((lane * 3 + j) & 1); }
  f32x4_peak_t acc[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) acc[q] = f32x4_peak_t{0.f, 0.f, 0.f, 0.f};
  uint32_t v[K > 0 ? K : 1];
#pragma unroll
  for (int j = 0; j < (K > 0 ? K : 1); ++j) v[j] = (uint32_t)(threadIdx.x * 17 + j);
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      acc[u & 3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, acc[u & 3], 0, 0, 0);
#pragma unroll
      for (int j = 0; j < K; ++j) asm volatile("v_xor_b32 %0, %0, %1" : "+v"(v[j]) : "v"(lane));
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e) s += acc[q][e];
  uint32_t r = 0;
#pragma unroll
  for (int j = 0; j < (K > 0 ? K : 1); ++j) r ^= v[j];
  if (s == -1.f) sink[0] = s + (float)r;  // never true (all products are >= 0): keeps the loops alive
}
