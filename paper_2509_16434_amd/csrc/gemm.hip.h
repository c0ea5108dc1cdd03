// bf16 MFMA tile kernels: C = A * B^T with pluggable A-row loaders (plain rows, implicit
// im2col of a 3x3 stride-2 pad-1 convolution, implicit col2im gather of its transpose) and
// pluggable epilogues, plus the weight-gradient kernel that contracts over rows.
//
// MFMA used: v_mfma_f32_32x32x16_bf16 (gfx950).  Operand layout per lane l of a wave:
//   A: row  l%32, k = (l/32)*8 .. +7      B: col l%32, k = (l/32)*8 .. +7
//   D: col  l%32, rows (e/4)*8 + (l/32)*4 + e%4 for e = 0..15
#pragma once
#include "common.hip.h"

#define GEMM_BK 32
#define GEMM_PITCH 40  // bf16 elements per LDS row (32 + 8 pad, keeps 16-byte alignment)

__device__ __forceinline__ uint4 zero16() { return make_uint4(0u, 0u, 0u, 0u); }

// ---------------------------------------------------------------- A-row loaders
// Rows of a channel-last tensor: row m = (img, q) with img = m / HW, q = m % HW, each row C
// elements wide, images addressed through ImgAddr (plain matrices: HW = 1, V = 1, stride_b = lda).
struct ARows {
  ImgAddr a; int HW, C, M, K;
  struct Row { const bf16_t* p; };
  __device__ __forceinline__ Row row(int m) const {
    Row r; r.p = nullptr;
    if (m < M) { int img = m / HW, q = m - img * HW; r.p = a.ptr(img) + (int64_t)q * C; }
    return r;
  }
  __device__ __forceinline__ uint4 load(const Row& r, int k) const {
    if (!r.p || k >= K) return zero16();
    return *reinterpret_cast<const uint4*>(r.p + k);
  }
};

// Row m = (img, oy, ox) of the im2col matrix of a channel-last image; k = (u*3+v)*Cin + ci.
struct AConvFwd {
  ImgAddr in; int H, W, Cin, Ho, Wo, M, K;
  struct Row { const bf16_t* p; int iy0, ix0; };
  __device__ __forceinline__ Row row(int m) const {
    Row r; r.p = nullptr; r.iy0 = 0; r.ix0 = 0;
    if (m < M) {
      int hw = Ho * Wo, img = m / hw, q = m - img * hw, oy = q / Wo, ox = q - oy * Wo;
      r.p = in.ptr(img); r.iy0 = 2 * oy - 1; r.ix0 = 2 * ox - 1;
    }
    return r;
  }
  __device__ __forceinline__ uint4 load(const Row& r, int k) const {
    if (!r.p || k >= K) return zero16();
    int tap = k / Cin, ci = k - tap * Cin, u = tap / 3, v = tap - 3 * u;
    int iy = r.iy0 + u, ix = r.ix0 + v;
    if ((unsigned)iy >= (unsigned)H || (unsigned)ix >= (unsigned)W) return zero16();
    return *reinterpret_cast<const uint4*>(r.p + ((int64_t)iy * W + ix) * Cin + ci);
  }
};

// Transposed convolution, one input-pixel parity class (py, px): rows are the input pixels
// (img, 2a+py, 2b+px); k = (tu*nv+tv)*Cout + co runs over the 1, 2 or 4 kernel taps that reach
// this class and the output channels.  Tap tu of an odd row is u = 2*tu (reads output row
// a+1-tu); an even row has the single tap u = 1 (output row a).  Same along x.
struct AConvDgrad {
  ImgAddr dy; int Ho, Wo, Cout, Ha, Wa, py, px, nv, M, K;
  struct Row { const bf16_t* p; int a, b; };
  __device__ __forceinline__ Row row(int m) const {
    Row r; r.p = nullptr; r.a = 0; r.b = 0;
    if (m < M) {
      int hw = Ha * Wa, img = m / hw, q = m - img * hw;
      r.a = q / Wa; r.b = q - r.a * Wa; r.p = dy.ptr(img);
    }
    return r;
  }
  __device__ __forceinline__ uint4 load(const Row& r, int k) const {
    if (!r.p || k >= K) return zero16();
    int t = k / Cout, co = k - t * Cout, tu = t / nv, tv = t - tu * nv;
    int oy = r.a + (py ? 1 - tu : 0), ox = r.b + (px ? 1 - tv : 0);
    if (oy >= Ho || ox >= Wo) return zero16();
    return *reinterpret_cast<const uint4*>(r.p + ((int64_t)oy * Wo + ox) * Cout + co);
  }
};

// ---------------------------------------------------------------- epilogues
// Output rows use the same (img, q) addressing as ARows; optional bias, ReLU, and a
// ReLU-derivative mask read from `mask` at the output's own offset.
template <typename OutT, bool BIAS, bool RELU, bool MASK>
struct EpRows {
  OutT* out; int64_t stride_b, stride_v; int V, HW, C; const float* bias; const bf16_t* mask; int M, N;
  __device__ __forceinline__ int64_t row_offset(int m) const {
    if (m >= M) return -1;
    int img = m / HW, q = m - img * HW, b = img / V, v = img - b * V;
    return (int64_t)b * stride_b + (int64_t)v * stride_v + (int64_t)q * C;
  }
  __device__ __forceinline__ void store(int64_t off, int n, float v) const {
    if (n >= N) return;
    if (BIAS) v += bias[n];
    if (RELU) v = v > 0.f ? v : 0.f;
    if (MASK) { if (!(bf2f(mask[off + n]) > 0.f)) v = 0.f; }
    if (sizeof(OutT) == 2) reinterpret_cast<bf16_t*>(out)[off + n] = f2bf(v);
    else reinterpret_cast<float*>(out)[off + n] = v;
  }
};

// Output rows are the input pixels of one parity class of a transposed convolution; the
// result is masked by the ReLU derivative of the activation stored at the same address.
struct EpConvDgrad {
  ImgAddrW out; ImgAddr act; int H, W, Cin, Ha, Wa, py, px, M;
  __device__ __forceinline__ int64_t row_offset(int m) const {
    if (m >= M) return -1;
    int hw = Ha * Wa, img = m / hw, q = m - img * hw, a = q / Wa, b = q - a * Wa;
    int64_t pix = ((int64_t)(2 * a + py) * W + (2 * b + px)) * Cin;
    // out and act share one addressing scheme; keep the image base in the offset
    return (out.ptr(img) - out.base) + pix;
  }
  __device__ __forceinline__ void store(int64_t off, int n, float v) const {
    if (n >= Cin) return;
    if (!(bf2f(act.base[off + n]) > 0.f)) v = 0.f;
    out.base[off + n] = f2bf(v);
  }
};

// ---------------------------------------------------------------- C = A * B^T
// B is a plain [N][K] matrix (row stride ldb).  256 threads = 4 waves laid out WGM x WGN, each
// computing TM x TN 32x32 MFMA tiles.  K is walked in steps of 32 through double-buffered LDS.
template <int BM, int BN, int WGM, int WGN, class AL, class EP>
__global__ __launch_bounds__(256) void k_gemm(AL al, const bf16_t* __restrict__ Bm, int64_t ldb, int N, int K, EP ep) {
  constexpr int TM = BM / (WGM * 32), TN = BN / (WGN * 32);
  static_assert(WGM * WGN == 4 && TM >= 1 && TN >= 1, "tile shape");
  constexpr int ACH = BM * 4 / 256, BCH = (BN * 4 + 255) / 256;  // 16-byte chunks per thread
  __shared__ __attribute__((aligned(16))) bf16_t As[2][BM * GEMM_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Bs[2][BN * GEMM_PITCH];
  __shared__ int64_t rowoff[BM];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;

  typename AL::Row arow[ACH];
  int a_r[ACH], a_k[ACH];
#pragma unroll
  for (int c = 0; c < ACH; ++c) {
    int ch = tid + c * 256;
    a_r[c] = ch >> 2; a_k[c] = (ch & 3) * 8;
    arow[c] = al.row(m0 + a_r[c]);
  }
  const bf16_t* brow[BCH]; int b_r[BCH], b_k[BCH];
#pragma unroll
  for (int c = 0; c < BCH; ++c) {
    int ch = tid + c * 256;
    b_r[c] = ch >> 2; b_k[c] = (ch & 3) * 8;
    int n = n0 + b_r[c];
    brow[c] = (b_r[c] < BN && n < N) ? Bm + (int64_t)n * ldb : nullptr;
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[ACH], rb[BCH];
  auto gload = [&](int k0) {
#pragma unroll
    for (int c = 0; c < ACH; ++c) ra[c] = al.load(arow[c], k0 + a_k[c]);
#pragma unroll
    for (int c = 0; c < BCH; ++c) {
      int k = k0 + b_k[c];
      rb[c] = (brow[c] && k < K) ? *reinterpret_cast<const uint4*>(brow[c] + k) : zero16();
    }
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < ACH; ++c) *reinterpret_cast<uint4*>(&As[buf][a_r[c] * GEMM_PITCH + a_k[c]]) = ra[c];
#pragma unroll
    for (int c = 0; c < BCH; ++c)
      if (b_r[c] < BN) *reinterpret_cast<uint4*>(&Bs[buf][b_r[c] * GEMM_PITCH + b_k[c]]) = rb[c];
  };

  const int nk = (K + GEMM_BK - 1) / GEMM_BK;
  gload(0);
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nk) gload((kt + 1) * GEMM_BK);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      bf16x8_t a[TM], b[TN];
      const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8_t*>(&As[buf][((wm * TM + i) * 32 + (lane & 31)) * GEMM_PITCH + kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8_t*>(&Bs[buf][((wn * TN + j) * 32 + (lane & 31)) * GEMM_PITCH + kk]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) sstore(buf ^ 1);
    __syncthreads();
  }

  for (int r = tid; r < BM; r += 256) rowoff[r] = ep.row_offset(m0 + r);
  __syncthreads();
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int rl = (wm * TM + i) * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        const int64_t off = rowoff[rl];
        if (off >= 0) ep.store(off, col, acc[i][j][e]);
      }
    }
}

// ---------------------------------------------------------------- weight gradient
// G[n][k] (+)= sum_m Dy[m][n] * A[m][k]: both operands are row-major over the contracted index m,
// so 16-byte chunks (8 consecutive n or k of one row m) are written transposed into LDS and the
// MFMA operands are then read as 8 consecutive m.  Block tile 64 (n) x 64 (k), 32 rows of m per
// step; grid.z splits the m range, each split writing its own fp32 partial tile (summed later in
// a fixed order).  Block (x == 0) also accumulates the column sums of Dy (the bias gradient).
template <class DL, class AL>
__global__ __launch_bounds__(256) void k_wgrad(DL dl, AL al, int Nn, int Kk, int M, int rows_per_split,
                                               float* __restrict__ partial, float* __restrict__ bias_partial) {
  __shared__ __attribute__((aligned(16))) bf16_t Ds[2][64 * GEMM_PITCH];
  __shared__ __attribute__((aligned(16))) bf16_t Xs[2][64 * GEMM_PITCH];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wn = wave >> 1, wk = wave & 1;
  const int k0 = blockIdx.x * 64, n0 = blockIdx.y * 64;
  const int split = blockIdx.z;
  const int mbeg = split * rows_per_split;
  const int mend = min(M, mbeg + rows_per_split);
  const int ml = tid & 31, g8 = (tid >> 5) * 8;  // this thread's row within the step and its 8-wide column group

  f32x16_t acc;
#pragma unroll
  for (int e = 0; e < 16; ++e) acc[e] = 0.f;
  float bsum = 0.f;

  uint4 rd, rx;
  auto gload = [&](int mb) {
    int m = mb + ml;
    bool ok = m < mend;
    typename DL::Row dr = dl.row(ok ? m : M);
    typename AL::Row ar = al.row(ok ? m : M);
    rd = dl.load(dr, n0 + g8);
    rx = al.load(ar, k0 + g8);
  };
  auto sstore = [&](int buf) {
    const bf16_t* d = reinterpret_cast<const bf16_t*>(&rd);
    const bf16_t* x = reinterpret_cast<const bf16_t*>(&rx);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      Ds[buf][(g8 + j) * GEMM_PITCH + ml] = d[j];
      Xs[buf][(g8 + j) * GEMM_PITCH + ml] = x[j];
    }
  };
  const int nsteps = (mend > mbeg) ? (mend - mbeg + 31) / 32 : 0;
  if (nsteps > 0) { gload(mbeg); sstore(0); }
  __syncthreads();
  for (int st = 0; st < nsteps; ++st) {
    const int buf = st & 1;
    if (st + 1 < nsteps) gload(mbeg + (st + 1) * 32);
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int kk = ks * 16 + (lane >> 5) * 8;
      bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(&Ds[buf][(wn * 32 + (lane & 31)) * GEMM_PITCH + kk]);
      bf16x8_t b = *reinterpret_cast<const bf16x8_t*>(&Xs[buf][(wk * 32 + (lane & 31)) * GEMM_PITCH + kk]);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
    if (bias_partial && blockIdx.x == 0 && tid < 64) {
      const bf16_t* r = &Ds[buf][tid * GEMM_PITCH];
#pragma unroll
      for (int m = 0; m < 32; ++m) bsum += bf2f(r[m]);
    }
    if (st + 1 < nsteps) sstore(buf ^ 1);
    __syncthreads();
  }
  float* P = partial + (int64_t)split * Nn * Kk;
  const int k = k0 + wk * 32 + (lane & 31);
#pragma unroll
  for (int e = 0; e < 16; ++e) {
    const int n = n0 + wn * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
    if (n < Nn && k < Kk) P[(int64_t)n * Kk + k] = acc[e];
  }
  if (bias_partial && blockIdx.x == 0 && tid < 64 && n0 + tid < Nn) bias_partial[(int64_t)split * Nn + n0 + tid] = bsum;
}

// dst[i] = (accumulate ? dst[i] : 0) + sum_s partial[s][i]; four interleaved running sums
// (s mod 4) combined as (s0+s1)+(s2+s3), always in the same order.
__global__ void k_reduce_partials(const float* __restrict__ partial, int splits, int64_t n, float* __restrict__ dst,
                                  int accumulate) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int k = 0;
  for (; k + 4 <= splits; k += 4) {
    s0 += partial[(int64_t)k * n + i]; s1 += partial[(int64_t)(k + 1) * n + i];
    s2 += partial[(int64_t)(k + 2) * n + i]; s3 += partial[(int64_t)(k + 3) * n + i];
  }
  for (; k < splits; ++k) s0 += partial[(int64_t)k * n + i];
  float s = (s0 + s1) + (s2 + s3);
  dst[i] = accumulate ? dst[i] + s : s;
}
