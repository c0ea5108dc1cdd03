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
// A loader describes the rows of the A matrix of an implicit GEMM, split so that nothing that
// depends on the row alone or on the column alone is recomputed per fetch:
//   cls(z)                    per-grid.z parameter set (row count M, depth K, weight matrix)
//   row(m, cls) -> Row        the row's base address, pixel offset and tap-validity bits
//   advance(Row&, delta, m)   the row delta further on (weight-gradient kernel)
//   kcur(k, cls) -> KCur      the column's tap / channel / element offset (k a multiple of 8)
//   kstep(KCur&, dk, cls)     the column dk further on
//   addr(Row, KCur, cls)      address of A[m][k..k+7], nullptr where those are zeros
// prepare() (host) fills the division constants from the geometry fields.

// Rows of a channel-last tensor: row m = (img, q) with img = m / HW, q = m % HW, each row C
// elements wide, images addressed through ImgAddr (plain matrices: HW = 1, V = 1, stride_b = lda).
struct ARows {
  ImgAddr a; int HW, C, M, K;
  bool plain;  // HW == 1, one view, no gather: consecutive rows are stride_b apart
  FastDiv dhw;
  void prepare() { a.prepare(); dhw = make_fastdiv(HW); }
  struct Row { const bf16_t* p; int img, q; };
  struct KCur { int k; };
  struct Cls { int M, K; };
  __device__ __forceinline__ Cls cls(int) const { Cls c; c.M = M; c.K = K; return c; }
  __device__ __forceinline__ const bf16_t* bmat(const Cls&, const bf16_t* dflt) const { return dflt; }
  __device__ __forceinline__ Row row(int m, const Cls&) const { return row(m); }
  __device__ __forceinline__ Row row(int m) const {
    Row r; r.p = nullptr; r.img = 0; r.q = 0;
    if (m < M) {
      if (plain) { r.img = m; r.p = a.base + (int64_t)m * a.stride_b; }
      else { r.img = (int)dhw.div((uint32_t)m); r.q = m - r.img * HW; r.p = a.ptr(r.img) + (int64_t)r.q * C; }
    }
    return r;
  }
  __device__ __forceinline__ void advance(Row& r, int delta, int m_new) const {
    if (m_new >= M) { r.p = nullptr; return; }
    if (plain) { r.p += (int64_t)delta * a.stride_b; return; }
    r.q += delta;
    if (r.q < HW) { r.p += (int64_t)delta * C; return; }
    while (r.q >= HW) { r.q -= HW; ++r.img; }
    r.p = a.ptr(r.img) + (int64_t)r.q * C;
  }
  __device__ __forceinline__ KCur kcur(int k, const Cls&) const { KCur c; c.k = k; return c; }
  __device__ __forceinline__ void kstep(KCur& c, int dk, const Cls&) const { c.k += dk; }
  __device__ __forceinline__ const bf16_t* addr(const Row& r, const KCur& c, const Cls&) const {
    return (!r.p || c.k >= K) ? nullptr : r.p + c.k;
  }
};

// Row m = (img, oy, ox) of the im2col matrix of a channel-last image under a 3x3 stride-2 pad-1
// window; k = (u*3+v)*Cin + ci.  Cin is a power of two (lc = log2 Cin).  A row keeps the element
// offset of its window's corner pixel (iy0, ix0) = (2oy-1, 2ox-1), which may lie outside the
// image, and one validity bit per tap; a column keeps its tap and the tap's element offset.
struct AConvFwd {
  ImgAddr in; int H, W, Cin, lc, Ho, Wo, M, K;
  FastDiv dhw, dwo;
  void prepare() { in.prepare(); dhw = make_fastdiv(Ho * Wo); dwo = make_fastdiv(Wo); }
  struct Row { const bf16_t* base; int poff, iy0, ix0, img; uint32_t vm; };
  struct KCur { int tap, ci, off; };
  struct Cls { int M, K; };
  __device__ __forceinline__ Cls cls(int) const { Cls c; c.M = M; c.K = K; return c; }
  __device__ __forceinline__ const bf16_t* bmat(const Cls&, const bf16_t* dflt) const { return dflt; }
  __device__ __forceinline__ void finish(Row& r) const {
    r.poff = (r.iy0 * W + r.ix0) << lc;
    const uint32_t cv = (r.ix0 >= 0 ? 1u : 0u) | 2u | (r.ix0 + 2 < W ? 4u : 0u);  // taps v = 0, 1, 2
    r.vm = (r.iy0 >= 0 ? cv : 0u) | (cv << 3) | (r.iy0 + 2 < H ? (cv << 6) : 0u);
  }
  __device__ __forceinline__ Row row(int m, const Cls&) const { return row(m); }
  __device__ __forceinline__ Row row(int m) const {
    Row r; r.base = nullptr; r.poff = 0; r.iy0 = 0; r.ix0 = 0; r.img = 0; r.vm = 0u;
    if (m < M) {
      const int hw = Ho * Wo, img = (int)dhw.div((uint32_t)m), q = m - img * hw;
      const int oy = (int)dwo.div((uint32_t)q), ox = q - oy * Wo;
      r.base = in.ptr(img); r.iy0 = 2 * oy - 1; r.ix0 = 2 * ox - 1; r.img = img;
      finish(r);
    }
    return r;
  }
  __device__ __forceinline__ void advance(Row& r, int delta, int m_new) const {
    if (m_new >= M) { r.base = nullptr; r.vm = 0u; return; }
    r.ix0 += 2 * delta;
    if (r.ix0 >= 2 * Wo - 1) {
      while (r.ix0 >= 2 * Wo - 1) { r.ix0 -= 2 * Wo; r.iy0 += 2; }
      if (r.iy0 >= 2 * Ho - 1) {
        while (r.iy0 >= 2 * Ho - 1) { r.iy0 -= 2 * Ho; ++r.img; }
        r.base = in.ptr(r.img);
      }
    }
    finish(r);
  }
  __device__ __forceinline__ void set_off(KCur& c) const {
    const int u = (c.tap * 11) >> 5, v = c.tap - 3 * u;  // tap / 3 for tap < 32
    c.off = ((u * W + v) << lc) + c.ci;
  }
  __device__ __forceinline__ KCur kcur(int k, const Cls&) const {
    KCur c; c.tap = k >> lc; c.ci = k & (Cin - 1); set_off(c); return c;
  }
  __device__ __forceinline__ void kstep(KCur& c, int dk, const Cls&) const {
    c.ci += dk; c.tap += c.ci >> lc; c.ci &= Cin - 1; set_off(c);
  }
  __device__ __forceinline__ const bf16_t* addr(const Row& r, const KCur& c, const Cls&) const {
    return ((r.vm >> (c.tap & 31)) & 1u) ? r.base + (r.poff + c.off) : nullptr;  // vm has no bits beyond tap 8
  }
};

// Transposed convolution.  A row is a horizontal PAIR of input pixels (img, iy, 2b), (img, iy, 2b+1)
// with iy = 2a+py and the row parity py selected by grid.z; its 2*Cin outputs are contiguous in
// memory (full 128-byte lines for Cin = 32).  The pair receives from output columns ox = b and
// b+1 (contiguous 2*Cout elements of dY) and from output rows oy = a (tap u = 1 for an even row;
// u = 2 for an odd row) and oy = a+1 (u = 0, odd rows only), so k = (tu*2 + dx)*Cout + co with tu
// over the 1 or 2 row taps and dx over the two columns.  The packed weight matrix of the parity
// holds zeros where a (pixel, column) combination has no tap (even pixel with dx = 1).
struct AConvDgrad {
  ImgAddr dy; int Ho, Wo, Cout, lco, H, W, dy_imgs;
  const bf16_t *w0, *w1;  // packed weights [2*Cin][nu*2*Cout] of row parity 0 / 1
  FastDiv dhw[2], dwb;
  void prepare() {
    dy.prepare();
    const int Wb = (W + 1) >> 1;
    dwb = make_fastdiv(Wb);
    for (int z = 0; z < 2; ++z) { const int Ha = (H - z + 1) >> 1; dhw[z] = make_fastdiv(Ha * Wb > 0 ? Ha * Wb : 1); }
  }
  struct Row { const bf16_t* base; int poff, a, b; uint32_t vm; };
  struct KCur { int t, co, off; };
  struct Cls { int Ha, Wb, py, M, K; const bf16_t* w; FastDiv dhw; };
  __device__ __forceinline__ Cls cls(int z) const {
    Cls c; c.py = z;
    c.Ha = (H - z + 1) >> 1; c.Wb = (W + 1) >> 1;
    c.M = dy_imgs * c.Ha * c.Wb; c.K = (1 + z) << (lco + 1);
    c.w = z ? w1 : w0;
    c.dhw = z ? dhw[1] : dhw[0];
    return c;
  }
  __device__ __forceinline__ const bf16_t* bmat(const Cls& c, const bf16_t*) const { return c.w; }
  __device__ __forceinline__ Row row(int m, const Cls& c) const {
    Row r; r.base = nullptr; r.poff = 0; r.a = 0; r.b = 0; r.vm = 0u;
    if (m < c.M) {
      const int hw = c.Ha * c.Wb, img = (int)c.dhw.div((uint32_t)m), q = m - img * hw;
      r.a = (int)dwb.div((uint32_t)q); r.b = q - r.a * c.Wb; r.base = dy.ptr(img);
      r.poff = (r.a * Wo + r.b) << lco;
      const uint32_t cx = 1u | (r.b + 1 < Wo ? 2u : 0u);  // dx = 0, 1
      // even rows: one row tap (oy = a); odd rows: tu = 0 -> oy = a+1, tu = 1 -> oy = a
      r.vm = c.py ? ((r.a + 1 < Ho ? cx : 0u) | (cx << 2)) : cx;
    }
    return r;
  }
  __device__ __forceinline__ void set_off(KCur& k, const Cls& c) const {
    const int tu = k.t >> 1, dx = k.t & 1;
    k.off = (((c.py ? 1 - tu : 0) * Wo + dx) << lco) + k.co;
  }
  __device__ __forceinline__ KCur kcur(int kk, const Cls& c) const {
    KCur k; k.t = kk >> lco; k.co = kk & (Cout - 1); set_off(k, c); return k;
  }
  __device__ __forceinline__ void kstep(KCur& k, int dk, const Cls& c) const {
    k.co += dk; k.t += k.co >> lco; k.co &= Cout - 1; set_off(k, c);
  }
  __device__ __forceinline__ const bf16_t* addr(const Row& r, const KCur& k, const Cls&) const {
    return ((r.vm >> (k.t & 31)) & 1u) ? r.base + (r.poff + k.off) : nullptr;  // vm has no bits beyond the parity's taps
  }
};

template <class AL>
__device__ __forceinline__ uint4 a_load(const AL& al, const typename AL::Row& r, const typename AL::KCur& c, const typename AL::Cls& cls) {
  const bf16_t* p = al.addr(r, c, cls);
  return p ? *reinterpret_cast<const uint4*>(p) : zero16();
}

// ---------------------------------------------------------------- epilogues
// Output row addressing: the same (img, q) scheme as ARows ...
struct MapRows {
  int64_t stride_b, stride_v; int V, HW, C, M;
  FastDiv dhw, dv;
  void prepare() { dhw = make_fastdiv(HW); dv = make_fastdiv(V); }
  struct Cls {};
  __device__ __forceinline__ Cls cls(int) const { return Cls(); }
  __device__ __forceinline__ int64_t row_offset(int m, const Cls&) const {
    if (m >= M) return -1;
    if (HW == 1 && V == 1) return (int64_t)m * stride_b;
    const int img = (int)dhw.div((uint32_t)m), q = m - img * HW, b = (int)dv.div((uint32_t)img), v = img - b * V;
    return (int64_t)b * stride_b + (int64_t)v * stride_v + (int64_t)q * C;
  }
  __device__ __forceinline__ int row_cols(int, const Cls&) const { return 0x7fffffff; }
};
// ... or horizontal pixel pairs of the rows of one parity of a transposed convolution's input.
struct MapDgrad {
  int64_t stride_b, stride_v; int V, H, W, Cin, imgs;
  FastDiv dhw[2], dwb, dv;
  void prepare() {
    const int Wb = (W + 1) >> 1;
    dwb = make_fastdiv(Wb); dv = make_fastdiv(V);
    for (int z = 0; z < 2; ++z) { const int Ha = (H - z + 1) >> 1; dhw[z] = make_fastdiv(Ha * Wb > 0 ? Ha * Wb : 1); }
  }
  struct Cls { int Ha, Wb, py, M; FastDiv dhw; };
  __device__ __forceinline__ Cls cls(int z) const {
    Cls c; c.py = z; c.Ha = (H - z + 1) >> 1; c.Wb = (W + 1) >> 1; c.M = imgs * c.Ha * c.Wb;
    c.dhw = z ? dhw[1] : dhw[0];
    return c;
  }
  __device__ __forceinline__ int64_t row_offset(int m, const Cls& c) const {
    if (m >= c.M) return -1;
    const int hw = c.Ha * c.Wb, img = (int)c.dhw.div((uint32_t)m), q = m - img * hw;
    const int a = (int)dwb.div((uint32_t)q), bb = q - a * c.Wb, b = (int)dv.div((uint32_t)img), v = img - b * V;
    return (int64_t)b * stride_b + (int64_t)v * stride_v + ((int64_t)(2 * a + c.py) * W + 2 * bb) * Cin;
  }
  // number of valid columns of the row: the last pair of an odd-width image has one pixel
  __device__ __forceinline__ int row_cols(int m, const Cls& c) const {
    const int bb = m - (int)dwb.div((uint32_t)m) * c.Wb;
    return (2 * bb + 1 < W) ? 2 * Cin : Cin;
  }
};
// out[off + n] = f(acc): optional bias, ReLU, and ReLU-derivative mask read from `mask` at the
// output's own offset (the stored activation whose gradient is being formed).  With `mbits` set the
// mask comes from the sign-bit words the forward kernel left instead (one bit per element, a
// sixteenth of the bytes): bit (off + n) of the bit string; the output must then be dense.
template <class MAP, typename OutT, bool BIAS, bool RELU, bool MASK>
struct Ep {
  typedef OutT out_t;
  static constexpr bool kBias = BIAS, kRelu = RELU, kMask = MASK;
  MAP map; OutT* out; const float* bias; const bf16_t* mask; int N;
  const uint32_t* mbits = nullptr;
};
// all-ones halves of a bf16 pair for the set bits among bits (2d, 2d + 1) of b
__device__ __forceinline__ uint32_t keep_halves(uint32_t b, int d) {
  return ((b >> (2 * d)) & 1u ? 0x0000ffffu : 0u) | ((b >> (2 * d + 1)) & 1u ? 0xffff0000u : 0u);
}

// Epilogue shared by the tile kernels.  acc[i][j][g*4+q] = C[m][n] with m = m0 + (wm*TM+i)*32 +
// lane%32, n = n0 + (wn*TN+j)*32 + g*8 + (lane/32)*4 + q.  bf16 results are packed four at a
// time, staged through `stage` (BM x (BN+8) elements of LDS no longer in use) and leave as
// 16-byte row segments; fp32 results are written directly.
// NTHR threads take part (all of them reach the barrier inside); waves without accumulators
// (has_acc false) only help to write the staged tile out.
template <int BM, int BN, int TM, int TN, int NTHR = 256, class EP, class MCLS>
__device__ __forceinline__ void gemm_epilogue(f32x16_t (&acc)[TM][TN], const EP& ep, const MCLS& mcls, int m0, int n0, int N, int wm, int wn,
                                              bf16_t* stage, int64_t* rowoff, int* rowcols, bool has_acc = true) {
  constexpr int SP = BN + 8;
  const int tid = threadIdx.x, lane = tid & 63;
  // acc[i][j][g*4+q] = C[m][n] with m = m0 + (wm*TM+i)*32 + lane%32, n = n0 + (wn*TN+j)*32 + g*8 + (lane/32)*4 + q
  typedef typename EP::out_t OutT;
  if constexpr (sizeof(OutT) == 2) {
    for (int r = tid; r < BM; r += NTHR) { rowoff[r] = ep.map.row_offset(m0 + r, mcls); rowcols[r] = ep.map.row_cols(m0 + r, mcls); }
    if (has_acc) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = (wn * TN + j) * 32 + g * 8 + (lane >> 5) * 4, nb = n0 + cl;
        float4 bv = make_float4(0.f, 0.f, 0.f, 0.f);
        if (EP::kBias) { if (nb < N) bv = *reinterpret_cast<const float4*>(ep.bias + nb); }  // N is a multiple of 8
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          float v0 = acc[i][j][g * 4] + bv.x, v1 = acc[i][j][g * 4 + 1] + bv.y, v2 = acc[i][j][g * 4 + 2] + bv.z, v3 = acc[i][j][g * 4 + 3] + bv.w;
          if (EP::kRelu) { v0 = fmaxf(v0, 0.f); v1 = fmaxf(v1, 0.f); v2 = fmaxf(v2, 0.f); v3 = fmaxf(v3, 0.f); }
          uint2 o; o.x = pack2bf(v0, v1); o.y = pack2bf(v2, v3);
          *reinterpret_cast<uint2*>(&stage[((wm * TM + i) * 32 + (lane & 31)) * SP + cl]) = o;
        }
      }
    }
    __syncthreads();
    constexpr int CPR = BN / 8;  // 16-byte chunks per row
    bf16_t* out = reinterpret_cast<bf16_t*>(ep.out);
    for (int ch = tid; ch < BM * CPR; ch += NTHR) {
      const int rl = ch / CPR, cg = ch - rl * CPR, n = n0 + cg * 8;
      const int64_t off = rowoff[rl];
      if (off < 0 || n >= N || n >= rowcols[rl]) continue;
      uint4 v = *reinterpret_cast<const uint4*>(&stage[rl * SP + cg * 8]);
      if (EP::kMask && ep.mbits) {
        const int64_t bi = off + n;  // a multiple of 8
        const uint32_t b = (ep.mbits[bi >> 5] >> (bi & 31)) & 0xffu;
        v.x &= keep_halves(b, 0); v.y &= keep_halves(b, 1); v.z &= keep_halves(b, 2); v.w &= keep_halves(b, 3);
      } else if (EP::kMask) {
        // keep a half where the stored activation is > 0 (sign bit clear and not zero)
        const uint4 mk = *reinterpret_cast<const uint4*>(ep.mask + off + n);
        auto keep = [](uint32_t m) -> uint32_t {
          return (((short)(m & 0xffffu) > 0) ? 0x0000ffffu : 0u) | (((short)(m >> 16) > 0) ? 0xffff0000u : 0u);
        };
        v.x &= keep(mk.x); v.y &= keep(mk.y); v.z &= keep(mk.z); v.w &= keep(mk.w);
      }
      if (EP::kMask) store_stream16(out + off + n, v);  // an activation gradient: large, read once by the layer below
      else *reinterpret_cast<uint4*>(out + off + n) = v;
    }
  } else {
    float* out = reinterpret_cast<float*>(ep.out);
    if (!has_acc) return;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int64_t off = ep.map.row_offset(m0 + (wm * TM + i) * 32 + (lane & 31), mcls);
      if (off < 0) continue;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int nb = n0 + (wn * TN + j) * 32 + g * 8 + (lane >> 5) * 4;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            if (nb + q >= N) continue;
            float x = acc[i][j][g * 4 + q];
            if (EP::kBias) x += ep.bias[nb + q];
            if (EP::kRelu) x = x > 0.f ? x : 0.f;
            if (EP::kMask) { if (!((short)ep.mask[off + nb + q] > 0)) x = 0.f; }
            out[off + nb + q] = x;
          }
        }
    }
  }
}

// ---------------------------------------------------------------- C = A * B^T
// B is a plain [N][K] matrix (row stride ldb; loaders with per-class weights override it).  256
// threads = 4 waves laid out WGM x WGN, each computing TM x TN 32x32 MFMA tiles.  K is walked in
// steps of 32 through double-buffered LDS.  The MFMA is issued with the weight tile as its first
// operand, so a lane ends up holding, for ONE output row m, four groups of four consecutive
// columns n.  bf16 results are packed four at a time, staged through LDS (8-byte writes) and
// leave as 16-byte row segments (with the ReLU mask read the same way); fp32 results are written
// directly.
template <int BM, int BN, int WGM, int WGN, int BK, class AL, class EP>
__global__ __launch_bounds__(256) void k_gemm(AL al, const bf16_t* __restrict__ Bm_, int64_t ldb_, int N, EP ep) {
  // BK = 32: double-buffered LDS, one barrier per step.  BK = 64: single LDS buffer with the next
  // step's tiles held in registers (twice the bytes in flight per block at the same LDS footprint).
  constexpr int TM = BM / (WGM * 32), TN = BN / (WGN * 32);
  static_assert(WGM * WGN == 4 && TM >= 1 && TN >= 1 && (BK == 32 || BK == 64), "tile shape");
  constexpr int CPK = BK / 8;                     // 16-byte chunks per row
  constexpr int PITCH = BK + 8, NBUF = (BK == 32) ? 2 : 1;
  constexpr int ACH = (BM * CPK + 255) / 256, BCH = (BN * CPK + 255) / 256;  // chunks per thread
  constexpr int AB_ELEMS = NBUF * (BM + BN) * PITCH;
  constexpr int SP = BN + 8;  // staging pitch (bf16 elements)
  static_assert(BM * SP <= AB_ELEMS, "staging tile must fit in the operand buffers");
  __shared__ __attribute__((aligned(16))) bf16_t smem[AB_ELEMS];
  __shared__ int64_t rowoff[BM];
  __shared__ int rowcols[BM];
  bf16_t* As = smem;                          // [NBUF][BM*PITCH]
  bf16_t* Bs = smem + NBUF * BM * PITCH;      // [NBUF][BN*PITCH]

  const typename AL::Cls acls = al.cls(blockIdx.z);
  const auto mcls = ep.map.cls(blockIdx.z);
  const int m0 = blockIdx.x * BM, n0 = blockIdx.y * BN;
  if (m0 >= acls.M) return;
  const int K = acls.K;
  const bf16_t* Bm = al.bmat(acls, Bm_);
  const int64_t ldb = (Bm == Bm_) ? ldb_ : (int64_t)K;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  // every chunk of a thread sits in the same 8-wide column group (256 is a multiple of CPK)
  const int ck = (tid % CPK) * 8;
  typename AL::Row arow[ACH];
  int a_r[ACH];
#pragma unroll
  for (int c = 0; c < ACH; ++c) {
    a_r[c] = (tid + c * 256) / CPK;
    arow[c] = al.row(a_r[c] < BM ? m0 + a_r[c] : acls.M, acls);
  }
  typename AL::KCur acur = al.kcur(ck, acls);
  const bf16_t* brow[BCH]; int b_r[BCH];
#pragma unroll
  for (int c = 0; c < BCH; ++c) {
    b_r[c] = (tid + c * 256) / CPK;
    int n = n0 + b_r[c];
    brow[c] = (b_r[c] < BN && n < N) ? Bm + (int64_t)n * ldb + ck : nullptr;
  }

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  uint4 ra[ACH], rb[BCH];
  int kb = 0;  // k of the tile being fetched
  auto gload = [&]() {
#pragma unroll
    for (int c = 0; c < ACH; ++c) ra[c] = a_load(al, arow[c], acur, acls);
#pragma unroll
    for (int c = 0; c < BCH; ++c) rb[c] = (brow[c] && kb + ck < K) ? *reinterpret_cast<const uint4*>(brow[c] + kb) : zero16();
    al.kstep(acur, BK, acls);
    kb += BK;
  };
  auto sstore = [&](int buf) {
#pragma unroll
    for (int c = 0; c < ACH; ++c)
      if (a_r[c] < BM) *reinterpret_cast<uint4*>(&As[buf * BM * PITCH + a_r[c] * PITCH + ck]) = ra[c];
#pragma unroll
    for (int c = 0; c < BCH; ++c)
      if (b_r[c] < BN) *reinterpret_cast<uint4*>(&Bs[buf * BN * PITCH + b_r[c] * PITCH + ck]) = rb[c];
  };

  const int nk = (K + BK - 1) / BK;
  gload();
  sstore(0);
  __syncthreads();
  for (int kt = 0; kt < nk; ++kt) {
    const int buf = (NBUF == 2) ? (kt & 1) : 0;
    if (kt + 1 < nk) gload();
    const bf16_t* Ab = As + buf * BM * PITCH;
    const bf16_t* Bb = Bs + buf * BN * PITCH;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8_t a[TM], b[TN];
      const int kk = ks * 16 + (lane >> 5) * 8;
#pragma unroll
      for (int i = 0; i < TM; ++i)
        a[i] = *reinterpret_cast<const bf16x8_t*>(&Ab[((wm * TM + i) * 32 + (lane & 31)) * PITCH + kk]);
#pragma unroll
      for (int j = 0; j < TN; ++j)
        b[j] = *reinterpret_cast<const bf16x8_t*>(&Bb[((wn * TN + j) * 32 + (lane & 31)) * PITCH + kk]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
    }
    if (NBUF == 1) __syncthreads();  // everyone is done reading the single buffer
    if (kt + 1 < nk) sstore(NBUF == 2 ? (buf ^ 1) : 0);
    __syncthreads();
  }

  gemm_epilogue<BM, BN, TM, TN>(acc, ep, mcls, m0, n0, N, wm, wn, smem, rowoff, rowcols);
}

// ---------------------------------------------------------------- weight gradient
// G[n][k] (+)= sum_m Dy[m][n] * A[m][k]: both operands are row-major over the contracted index m,
// while an MFMA lane needs 8 consecutive m of ONE column.  The tiles are stored in LDS as they
// come (16-byte row chunks, rows = m) and read back through ds_read_b64_tr_b16, which transposes
// within groups of 16 lanes: when lane r of a group supplies the address of 4 consecutive columns
// c0 + 4*(r%4) .. +3 of row m0 + r/4, lane i of the group receives column c0 + i of rows m0 .. m0+3.
// Two such reads give a lane its 8 m-values; the order of m inside the contraction is the same
// for both operands, which is all the sum needs.  Row pitches are 64 bytes mod 256, so the four
// rows a half-wave reads fall into disjoint banks.
//
// Block tile: 64 (n) x 128*KTW (k), 32 rows of m per step, double-buffered (one barrier per step);
// 8 consecutive lanes fetch 128 contiguous bytes of one row.  Wave w owns the k-tiles w, w+4, ...
// (KTW of them) for both 32-row n-tiles, so Dy is read once per 128*KTW columns of k.  grid.z splits
// the m range, each split writing its own fp32 partial tile (summed later in a fixed order).
// Block (x == 0) also accumulates the column sums of Dy (the bias gradient).  Rows are tracked
// incrementally (no integer division in the loop).
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8_t lds_read_tr8(const bf16_t* p, int rows4_elems) {
  // p: this lane's source address for the first 4 rows; the second 4 rows are rows4_elems further on
  struct { s16x4_t lo, hi; } v;
  v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p));
  v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t __attribute__((address_space(3)))*)(p + rows4_elems));
  return __builtin_bit_cast(bf16x8_t, v);
}

template <int KTW, class DL, class AL>
__global__ __launch_bounds__(256) void k_wgrad(DL dl, AL al, int Nn, int Kk, int M, int rows_per_split,
                                               float* __restrict__ partial, float* __restrict__ bias_partial) {
  constexpr int BKC = 128 * KTW;             // k columns per block
  constexpr int XCH = 2 * KTW;               // X chunks per thread per step
  constexpr int DP = 64 + 32, XP = BKC + 32; // row pitches (elements): 192 and 256*KTW + 64 bytes
  __shared__ __attribute__((aligned(16))) bf16_t Dt[2][32 * DP];
  __shared__ __attribute__((aligned(16))) bf16_t Xt[2][32 * XP];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int k0 = blockIdx.x * BKC, n0 = blockIdx.y * 64;
  const int split = blockIdx.z;
  const int mbeg = split * rows_per_split;
  const int mend = min(M, mbeg + rows_per_split);
  const int ml = tid >> 3, c8 = (tid & 7) * 8;  // this thread's row within the step and its first column
  const bool do_bias = bias_partial && blockIdx.x == 0;

  f32x16_t acc[KTW][2];
#pragma unroll
  for (int t = 0; t < KTW; ++t)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
  float bs[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) bs[j] = 0.f;

  int m = mbeg + ml;
  const typename DL::Cls dcls = dl.cls(0);
  const typename AL::Cls xcls = al.cls(0);
  typename DL::Row dr = dl.row(m < mend ? m : M);
  typename AL::Row ar = al.row(m < mend ? m : M);
  const typename DL::KCur dcur = dl.kcur(n0 + c8, dcls);  // this thread's columns never change
  typename AL::KCur xcur[XCH];
#pragma unroll
  for (int c = 0; c < XCH; ++c) xcur[c] = al.kcur(k0 + c * 64 + c8, xcls);
  uint4 rd, rx[XCH];
  auto gload = [&]() {
    const bool ok = m < mend;
    rd = ok ? a_load(dl, dr, dcur, dcls) : zero16();
#pragma unroll
    for (int c = 0; c < XCH; ++c) rx[c] = ok ? a_load(al, ar, xcur[c], xcls) : zero16();
  };
  auto sstore = [&](int buf) {
    *reinterpret_cast<uint4*>(&Dt[buf][ml * DP + c8]) = rd;
#pragma unroll
    for (int c = 0; c < XCH; ++c) *reinterpret_cast<uint4*>(&Xt[buf][ml * XP + c * 64 + c8]) = rx[c];
    if (do_bias) {
      bs[0] += bf2f((bf16_t)(rd.x & 0xffffu)); bs[1] += bf2f((bf16_t)(rd.x >> 16));
      bs[2] += bf2f((bf16_t)(rd.y & 0xffffu)); bs[3] += bf2f((bf16_t)(rd.y >> 16));
      bs[4] += bf2f((bf16_t)(rd.z & 0xffffu)); bs[5] += bf2f((bf16_t)(rd.z >> 16));
      bs[6] += bf2f((bf16_t)(rd.w & 0xffffu)); bs[7] += bf2f((bf16_t)(rd.w >> 16));
    }
  };
  // transposing reads: source row / column of this lane within a 16-row k-step and a 32-column tile
  const int g = lane >> 4, r16 = lane & 15;
  const int srow = 8 * (g >> 1) + (r16 >> 2), scol = 16 * (g & 1) + 4 * (r16 & 3);

  const int nsteps = (mend > mbeg) ? (mend - mbeg + 31) / 32 : 0;
  if (nsteps > 0) { gload(); sstore(0); }
  __syncthreads();
  for (int st = 0; st < nsteps; ++st) {
    const int buf = st & 1;
    if (st + 1 < nsteps) {
      m += 32;
      dl.advance(dr, 32, m < mend ? m : M);
      al.advance(ar, 32, m < mend ? m : M);
      gload();
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const bf16_t* dsrc = &Dt[buf][(ks * 16 + srow) * DP + scol];
      const bf16x8_t a0 = lds_read_tr8(dsrc, 4 * DP);
      const bf16x8_t a1 = lds_read_tr8(dsrc + 32, 4 * DP);
#pragma unroll
      for (int t = 0; t < KTW; ++t) {
        const int ktile = wave + 4 * t;
        if (k0 + ktile * 32 < Kk) {
          const bf16x8_t b = lds_read_tr8(&Xt[buf][(ks * 16 + srow) * XP + ktile * 32 + scol], 4 * XP);
          acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[t][0], 0, 0, 0);
          acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[t][1], 0, 0, 0);
        }
      }
    }
    if (st + 1 < nsteps) sstore(buf ^ 1);
    __syncthreads();
  }
  float* P = partial + (int64_t)split * Nn * Kk;
#pragma unroll
  for (int t = 0; t < KTW; ++t) {
    const int k = k0 + (wave + 4 * t) * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int n = n0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (n < Nn && k < Kk) P[(int64_t)n * Kk + k] = acc[t][i][e];
      }
  }
  if (do_bias) {
    // column sums: thread (row ml, columns c8..c8+7) -> sum over the 32 rows in a fixed order
    float* red = reinterpret_cast<float*>(&Xt[0][0]);  // 32 x 64 floats = 8 KB (the loop's last barrier has passed)
#pragma unroll
    for (int j = 0; j < 8; ++j) red[ml * 64 + c8 + j] = bs[j];
    __syncthreads();
    if (tid < 64 && n0 + tid < Nn) {
      float s = 0.f;
      for (int q = 0; q < 32; ++q) s += red[q * 64 + tid];
      bias_partial[(int64_t)split * Nn + n0 + tid] = s;
    }
  }
}

// Sum over s of partial[s][i .. i+W-1] for W (1 or 4) consecutive outputs per lane: a block covers
// 32*W outputs with 8 lanes of splits each (lane j sums s = j, j+8, ... with four running sums, four
// loads in flight); the 8 lane sums are combined in a fixed order, so the result does not depend on
// scheduling.  The sums are valid in the lanes with threadIdx.x < 32.
template <int W>
__device__ __forceinline__ void reduce_partials_block(const float* __restrict__ partial, int splits, int64_t n, int64_t i, float (*red)[33 * W], float (&out)[W]) {
  typedef float vec_t __attribute__((ext_vector_type(W)));
  const int o = threadIdx.x & 31, sl = threadIdx.x >> 5;
  vec_t s0 = 0.f, s1 = 0.f;
  if (i < n) {
    auto ld = [&](int k) -> vec_t { return *reinterpret_cast<const vec_t*>(partial + (int64_t)k * n + i); };
    int k = sl;
    vec_t s2 = 0.f, s3 = 0.f;
    for (; k + 24 < splits; k += 32) {
      const vec_t v0 = ld(k), v1 = ld(k + 8), v2 = ld(k + 16), v3 = ld(k + 24);
      s0 += v0; s1 += v1; s2 += v2; s3 += v3;
    }
    s0 += s2; s1 += s3;
    for (; k + 8 < splits; k += 16) { s0 += ld(k); s1 += ld(k + 8); }
    if (k < splits) s0 += ld(k);
  }
  s0 += s1;
#pragma unroll
  for (int w = 0; w < W; ++w) red[sl][o * W + w] = s0[w];
  __syncthreads();
#pragma unroll
  for (int w = 0; w < W; ++w) {
    const int c = o * W + w;
    out[w] = ((red[0][c] + red[1][c]) + (red[2][c] + red[3][c])) + ((red[4][c] + red[5][c]) + (red[6][c] + red[7][c]));
  }
}
