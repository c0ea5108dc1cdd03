// Fused backward of the first two convolutions: the transposed convolution of layer 1 (gradient
// w.r.t. the first layer's output) with the first layer's weight/bias gradient computed from the
// tile while it is still on chip.  The gradient w.r.t. the first layer's output has no other
// consumer (the image needs no gradient), so it is never written to HBM.
#pragma once
#include "gemm.hip.h"
#include "mem_kernels.hip.h"

// Persistent kernel: block b processes tiles b, b + gridDim.x, ... of 128 pixel-pair rows (both row
// parities, interleaved) and keeps its share of dW0[co][k] in MFMA accumulators across tiles.
//   1. dX tile = dY1-rows x packed transposed weights (as k_gemm with AConvDgrad), staged as bf16.
//   2. ReLU mask from the stored first-layer activation (16-byte row segments), written back to LDS.
//   3. dW0 += dX^T * patches: contraction over the tile's 256 pixels, 16 per MFMA; first operand
//      dX^T read transposed from LDS (lane: channel, 8 rows), second operand the 3x3 image patches
//      of those pixels, gathered once per tile from the rollout buffer (one thread per pixel) into
//      an LDS table [tap][pixel] (tap index K0 is the all-ones column giving the bias gradient).
// partial[block][C0*(K0+1)] is summed afterwards in block order.
template <int BN, int WGM, int WGN, int CIN0>
__global__ __launch_bounds__(256) void k_dgrad1_wgrad0(AConvDgrad al, MapDgrad map, const bf16_t* __restrict__ mask,
                                                       ImgAddr img_in, int H0, int W0, int tiles_per_parity,
                                                       float* __restrict__ partial) {
  constexpr int BM = 128, TM = BM / (WGM * 32), TN = BN / (WGN * 32);
  constexpr int BK = 64, PITCH = BK + 8, ACH = BM * (BK / 8) / 256;
  constexpr int SP = BN + 8;
  constexpr int SM_ELEMS = (BM * PITCH > BM * SP) ? BM * PITCH : BM * SP;
  constexpr int K0 = 9 * CIN0, KP1 = K0 + 1;
  __shared__ __attribute__((aligned(16))) bf16_t smem[SM_ELEMS];   // A tile, later the staged output tile
  __shared__ int64_t rowoff[BM];
  __shared__ int64_t rowbase[BM];
  __shared__ int rowyx[BM], rowcols[BM];
  constexpr int XR = (KP1 <= 16) ? 16 : 32, XP = 2 * BM + 8;  // patch table rows (taps, padded) and pitch
  __shared__ __attribute__((aligned(16))) bf16_t xT[XR * XP];
  // the packed transposed-conv weights of both row parities stay in LDS for the whole kernel, as
  // [k/8][BN][8] so that a lane's 8 consecutive k of column n are one conflict-free 16-byte read
  extern __shared__ __attribute__((aligned(16))) bf16_t wl[];
  bf16_t* As = smem;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int wm = wave / WGN, wn = wave % WGN;
  const int Cin = map.Cin, N = 2 * Cin, NJ = (Cin + 31) / 32;
  const int Kp0 = 2 << al.lco, Kp1 = 4 << al.lco;  // depth of parity 0 / 1
  for (int i = tid; i < (Kp0 + Kp1) / 8 * BN; i += 256) {
    const int k8 = i / BN, n = i - k8 * BN;
    uint4 v = zero16();
    if (n < N) v = (k8 < Kp0 / 8) ? *reinterpret_cast<const uint4*>(al.w0 + (int64_t)n * Kp0 + k8 * 8)
                                  : *reinterpret_cast<const uint4*>(al.w1 + (int64_t)n * Kp1 + (k8 - Kp0 / 8) * 8);
    *reinterpret_cast<uint4*>(&wl[(int64_t)i * 8]) = v;
  }
  // the patch table's unused rows stay zero for the whole kernel
  for (int i = tid; i < XR * XP; i += 256) xT[i] = 0;

  f32x16_t accw[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int e = 0; e < 16; ++e) accw[jn][e] = 0.f;

  for (int tile = blockIdx.x; tile < 2 * tiles_per_parity; tile += gridDim.x) {
    const int z = tile & 1, m0 = (tile >> 1) * BM;
    const AConvDgrad::Cls acls = al.cls(z);
    const MapDgrad::Cls mcls = map.cls(z);
    if (m0 >= acls.M) continue;  // block-uniform
    const int K = acls.K;
    const bf16_t* Wz = wl + (z ? (Kp0 / 8) * BN * 8 : 0);

    AConvDgrad::Row arow[ACH];
    int a_r[ACH];
    const int ck = (tid & 7) * 8;  // the same column group for all of a thread's chunks
#pragma unroll
    for (int c = 0; c < ACH; ++c) {
      a_r[c] = (tid + c * 256) >> 3;
      arow[c] = al.row(m0 + a_r[c], acls);
    }
    AConvDgrad::KCur acur = al.kcur(ck, acls);
    f32x16_t acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

    uint4 ra[ACH];
    auto gload = [&]() {
#pragma unroll
      for (int c = 0; c < ACH; ++c) ra[c] = a_load(al, arow[c], acur, acls);
      al.kstep(acur, BK, acls);
    };
    gload();
    __syncthreads();  // the previous tile's LDS readers are done
    // ---- 0. row tables, then issue the loads the epilogue will need (ReLU mask segments of the stored
    //         activation, this thread's image patch) so that their latency overlaps the main loop
    for (int r = tid; r < BM; r += 256) {
      const int m = m0 + r;
      int64_t off = -1, base = 0; int yx = 0, cols = 0;
      if (m < mcls.M) {
        const int hw = mcls.Ha * mcls.Wb, img = (int)mcls.dhw.div((uint32_t)m), q = m - img * hw;
        const int a = (int)map.dwb.div((uint32_t)q), bb = q - a * mcls.Wb;
        const int b = (int)map.dv.div((uint32_t)img), v = img - b * map.V;
        const int iy = 2 * a + mcls.py, ix0 = 2 * bb;
        off = (int64_t)b * map.stride_b + (int64_t)v * map.stride_v + ((int64_t)iy * map.W + ix0) * Cin;
        base = img_in.ptr(img) - img_in.base;
        yx = (iy << 16) | ix0;
        cols = (ix0 + 1 < map.W) ? 2 * Cin : Cin;
      }
      rowoff[r] = off; rowbase[r] = base; rowyx[r] = yx; rowcols[r] = cols;
    }
    __syncthreads();
    constexpr int CPR = BN / 8, MCH = BM * CPR / 256;
    uint4 mk[MCH];
#pragma unroll
    for (int c = 0; c < MCH; ++c) {
      const int ch = tid + c * 256, rl = ch / CPR, n = (ch - rl * CPR) * 8;
      const int64_t off = rowoff[rl];
      mk[c] = (off >= 0 && n < rowcols[rl]) ? *reinterpret_cast<const uint4*>(mask + off + n) : zero16();
    }
    bf16_t xv[KP1];
    {  // thread -> pixel (row r = tid % 128, px = tid / 128)
      const int r = tid & (BM - 1), px = tid >> 7;
      const int yx = rowyx[r], iy = yx >> 16, ix = (yx & 0xffff) + px;
      const bool ok = rowoff[r] >= 0 && ix < map.W;
      const bf16_t* pb = img_in.base + rowbase[r] + ((2 * iy - 1) * W0 + (2 * ix - 1)) * CIN0;
      const bool rok[3] = {iy > 0, true, 2 * iy + 1 < H0};
      const bool cok[3] = {ix > 0, true, 2 * ix + 1 < W0};
#pragma unroll
      for (int u = 0; u < 3; ++u)
#pragma unroll
        for (int v = 0; v < 3; ++v)
#pragma unroll
          for (int c = 0; c < CIN0; ++c)
            xv[(u * 3 + v) * CIN0 + c] = (ok && rok[u] && cok[v]) ? pb[(u * W0 + v) * CIN0 + c] : (bf16_t)0;
      xv[K0] = ok ? (bf16_t)0x3F80 : (bf16_t)0;  // 1.0
    }
    // ---- main loop: 64-wide k steps, A through one LDS buffer with the next step held in registers
    const int nk = (K + BK - 1) / BK;
    for (int kt = 0; kt < nk; ++kt) {
      if (kt > 0) __syncthreads();  // the previous step's readers are done
#pragma unroll
      for (int c = 0; c < ACH; ++c) *reinterpret_cast<uint4*>(&As[a_r[c] * PITCH + ck]) = ra[c];
      __syncthreads();
      if (kt + 1 < nk) gload();
#pragma unroll
      for (int ks = 0; ks < BK / 16; ++ks) {
        bf16x8_t a[TM], b[TN];
        const int kk = ks * 16 + h * 8;
#pragma unroll
        for (int i = 0; i < TM; ++i) a[i] = *reinterpret_cast<const bf16x8_t*>(&As[((wm * TM + i) * 32 + l32) * PITCH + kk]);
#pragma unroll
        for (int j = 0; j < TN; ++j)
          b[j] = (kt * BK + kk < K) ? *reinterpret_cast<const bf16x8_t*>(&Wz[(((kt * BK + kk) >> 3) * BN + (wn * TN + j) * 32 + l32) * 8])
                                    : __builtin_bit_cast(bf16x8_t, zero16());
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[j], a[i], acc[i][j], 0, 0, 0);
      }
    }
    __syncthreads();  // all waves are done with the A tile; its LDS becomes the staging tile

    // ---- 1. the unmasked bf16 tile
    bf16_t* stage = smem;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = (wn * TN + j) * 32 + g * 8 + h * 4;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          uint2 o; o.x = pack2bf(acc[i][j][g * 4], acc[i][j][g * 4 + 1]); o.y = pack2bf(acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
          *reinterpret_cast<uint2*>(&stage[((wm * TM + i) * 32 + l32) * SP + cl]) = o;
        }
      }
    __syncthreads();
    // ---- 2. ReLU mask of the stored first-layer activation (loaded at the top), applied in place
#pragma unroll
    for (int c = 0; c < MCH; ++c) {
      const int ch = tid + c * 256, rl = ch / CPR, n = (ch - rl * CPR) * 8;
      uint4 v = *reinterpret_cast<const uint4*>(&stage[rl * SP + n]);
      auto keep = [](uint32_t m) -> uint32_t {
        return (((short)(m & 0xffffu) > 0) ? 0x0000ffffu : 0u) | (((short)(m >> 16) > 0) ? 0xffff0000u : 0u);
      };
      // invalid rows / columns were loaded as zero mask words, which clear the value
      v.x &= keep(mk[c].x); v.y &= keep(mk[c].y); v.z &= keep(mk[c].z); v.w &= keep(mk[c].w);
      *reinterpret_cast<uint4*>(&stage[rl * SP + n]) = v;
    }
    // ---- 3. first-layer weight gradient from the tile
    // patch table column of this thread's pixel: px*128 + r = tid
#pragma unroll
    for (int k = 0; k < KP1; ++k) xT[k * XP + tid] = xv[k];
    __syncthreads();
    for (int g = wave; g < 8; g += 4) {  // 8 groups of 16 rows x the 2 pixels of the pair
#pragma unroll
      for (int px = 0; px < 2; ++px) {
        bf16x8_t xb;
        if (l32 < XR) xb = *reinterpret_cast<const bf16x8_t*>(&xT[l32 * XP + px * BM + g * 16 + h * 8]);
        else xb = __builtin_bit_cast(bf16x8_t, zero16());
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
          if (jn >= NJ) break;
          const int ci = jn * 32 + l32;
          bf16_t ds[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) ds[j] = (ci < Cin) ? stage[(g * 16 + h * 8 + j) * SP + px * Cin + ci] : (bf16_t)0;
          accw[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack8(ds), xb, accw[jn], 0, 0, 0);
        }
      }
    }
  }
  // ---- sum the four wave accumulators: accw[jn][g*4+q] = D[ci = jn*32 + g*8 + h*4 + q][k = l32]
  __syncthreads();
  float* wsum = reinterpret_cast<float*>(smem);  // [4][Cin*32] (the host checks that it fits)
  const int ws = Cin * 32;
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int ci = jn * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
      if (ci < Cin) wsum[wave * ws + ci * 32 + l32] = accw[jn][e];
    }
  __syncthreads();
  float* P = partial + (int64_t)blockIdx.x * Cin * KP1;
  for (int i = tid; i < Cin * KP1; i += 256) {
    const int co = i / KP1, k = i - co * KP1, s = co * 32 + k;
    P[i] = (wsum[s] + wsum[ws + s]) + (wsum[2 * ws + s] + wsum[3 * ws + s]);
  }
}
