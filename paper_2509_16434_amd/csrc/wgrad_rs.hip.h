// Weight gradient of a wide linear layer, G[n][k] (+)= sum over samples m of dY[m][n] * X[m][k]
// (plus the bias gradient, the column sums of dY), for plain row-major operands: the form of
// k_wgrad for large outputs (first hidden layer), organised like k_gemm_rs.
//
// A block owns a 128 (n) x 128 (k) tile of G and a range of samples.  Four loader waves bring
// 64 samples per stage into an LDS ring with LDS-writing 16-byte loads, as four blocks of
// [64 samples][64 columns] (128-byte rows): columns n0..+63, n0+64..+127 of dY and k0..+63,
// k0+64..+127 of X, one block per loader.  Four compute waves (64 x 64 of the tile each, 64
// accumulator registers) contract over the samples, 16 per MFMA step; both operands are read with
// transposing LDS reads from the row-major blocks (lane r of a 16-lane group supplies 4 consecutive
// columns of sample r/4; lane i receives column i of 4 samples).  Bit 6 of a block offset is
// flipped for every second pair of rows (by the loaders, through the source address), so that the
// four rows of one transposing read fall into different banks.  One barrier per stage.
//
// With one split the tile goes straight into the gradient (written or accumulated); with several,
// each split leaves an fp32 partial, summed afterwards in a fixed order.
#pragma once
#include "gemm_dma.hip.h"
#include "conv_tile.hip.h"

struct WgradRsArgs {
  const bf16_t* dy; int64_t ld_dy;  // [M][Nn]
  const bf16_t* x; int64_t ld_x;    // [M][Kk]
  int M, Nn, Kk, rows_per_split;    // Nn, Kk multiples of 8; rows_per_split a multiple of 64
  float* out;                       // direct: G [Nn][Kk]; else partial [splits][Nn][Kk]
  float* bias_out;                  // direct: gb [Nn]; else partial [splits][Nn]; NULL: no bias gradient
  int direct, accumulate;
  const bf16_t* zpage;              // 1 KiB of zeros
};

struct WgradRsShape {
  static constexpr int TN = 128, TK = 128, ROWS = 64, NST = 4, THREADS = 512;
  static constexpr int BLK_BYTES = ROWS * 128, ST_BYTES = 4 * BLK_BYTES, LDS_BYTES = NST * ST_BYTES;
};

__global__ __launch_bounds__(512) void k_wgrad_rs(WgradRsArgs a) {
  typedef WgradRsShape S;
  constexpr int NST = S::NST, D = NST - 1, BLK = S::BLK_BYTES, ST = S::ST_BYTES;
  extern __shared__ __attribute__((aligned(16))) char wring[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int k0 = blockIdx.x * S::TK, n0 = blockIdx.y * S::TN, split = blockIdx.z;
  const int mbeg = split * a.rows_per_split, mend = min(a.M, mbeg + a.rows_per_split);
  const int nst = mend > mbeg ? (mend - mbeg + S::ROWS - 1) / S::ROWS : 0;

  if (wave >= 4) {
    // ------------------------------------------------------------------ loaders: loader lw fills block lw of every stage
    const int lw = wave - 4;
    const bool is_x = lw >= 2;
    const bf16_t* base = is_x ? a.x : a.dy;
    const int64_t ld = is_x ? a.ld_x : a.ld_dy;
    const int col0 = (is_x ? k0 : n0) + (lw & 1) * 64, ncols = is_x ? a.Kk : a.Nn;
    const int dr = lane >> 3, dpos = lane & 7;
    // load j of a stage: rows j*8 + dr; LDS offset row*128 + dpos*16 holds the row's chunk dpos ^ 4*((row >> 1) & 1)
    const int col = col0 + ((dpos ^ (((dr >> 1) & 1) << 2)) * 8);
    const bool col_ok = col < ncols;
    const char* const zp = reinterpret_cast<const char*>(a.zpage) + lane * 16;
    const bf16_t* p0 = base + (int64_t)(mbeg + dr) * ld + col;  // row dr of the next stage to issue
    int m_next = mbeg + dr;
    auto issue = [&](int slot) __attribute__((always_inline)) {
      char* sb = wring + slot * ST + lw * BLK;
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const char* p = (col_ok && m_next + j * 8 < mend) ? reinterpret_cast<const char*>(p0 + (int64_t)(j * 8) * ld) : zp;
        __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(sb + j * 1024), 16, 0, 0);
      }
      p0 += (int64_t)S::ROWS * ld; m_next += S::ROWS;
    };
    int slot = 0;
    for (int s = 0; s < D && s < nst; ++s) { issue(slot); slot = slot == NST - 1 ? 0 : slot + 1; }
    for (int st = 0; st < nst; ++st) {
      const int younger = min(D - 1, nst - 1 - st);  // stages issued after stage st
      vm_wait_dyn(younger * 8);
      __builtin_amdgcn_s_barrier();  // stage st has landed; the compute waves have left stage st - 1
      if (st + D < nst) { issue(slot); slot = slot == NST - 1 ? 0 : slot + 1; }
    }
    return;
  }

  // -------------------------------------------------------------------- compute waves: 64 (n) x 64 (k) each
  const int wn = wave >> 1, wk = wave & 1;
  const int l32 = lane & 31, h = lane >> 5, g = lane >> 4, r16 = lane & 15;
  const int scolb = (16 * (g & 1) + 4 * (r16 & 3)) * 2;  // byte offset of this lane's 4 source columns in a 32-column tile
  uint32_t off[4][2];  // per MFMA step and half (samples +0..3 / +4..7 of the lane's group): source offset within a block, tile 0
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      const uint32_t dl = (uint32_t)((ks * 16 + 8 * (g >> 1) + (r16 >> 2) + 4 * hf) * 128 + scolb);
      off[ks][hf] = dl ^ (((dl >> 8) & 1u) << 6);
    }
  f32x16_t acc[2][2], accb[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
#pragma unroll
    for (int e = 0; e < 16; ++e) accb[i][e] = 0.f;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
  }
  const bool do_bias = a.bias_out && blockIdx.x == 0 && wk == 0;
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
  int slot = 0;
  for (int st = 0; st < nst; ++st) {
    __builtin_amdgcn_s_barrier();  // stage st is in LDS
    const char* ab = wring + slot * ST + wn * BLK;        // dY block of this wave's n half
    const char* xb = wring + slot * ST + (2 + wk) * BLK;  // X block of its k half
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8_t av[2], bv[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) av[i] = lds_read_tr8_2(ab + (off[ks][0] ^ (uint32_t)(i * 64)), ab + (off[ks][1] ^ (uint32_t)(i * 64)));
#pragma unroll
      for (int j = 0; j < 2; ++j) bv[j] = lds_read_tr8_2(xb + (off[ks][0] ^ (uint32_t)(j * 64)), xb + (off[ks][1] ^ (uint32_t)(j * 64)));
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], bv[j], acc[i][j], 0, 0, 0);
      if (do_bias) {
#pragma unroll
        for (int i = 0; i < 2; ++i) accb[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[i], ones, accb[i], 0, 0, 0);
      }
    }
    slot = slot == NST - 1 ? 0 : slot + 1;
  }
  // acc[i][j][e] = G[n][k], n = n0 + wn*64 + i*32 + (e/4)*8 + h*4 + e%4, k = k0 + wk*64 + j*32 + l32
  float* out = a.direct ? a.out : a.out + (int64_t)split * a.Nn * a.Kk;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int n = n0 + wn * 64 + i * 32 + (e >> 2) * 8 + h * 4 + (e & 3);
      if (n >= a.Nn) continue;
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const int k = k0 + wk * 64 + j * 32 + l32;
        if (k < a.Kk) {
          float* d = out + (int64_t)n * a.Kk + k;
          *d = (a.direct && a.accumulate) ? *d + acc[i][j][e] : acc[i][j][e];
        }
      }
      if (do_bias && l32 == 0) {
        float* d = a.direct ? a.bias_out + n : a.bias_out + (int64_t)split * a.Nn + n;
        *d = (a.direct && a.accumulate) ? *d + accb[i][e] : accb[i][e];
      }
    }
}
