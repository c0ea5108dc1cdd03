// First convolution (1 or 3 input channels -> up to 64 output channels, 3x3 stride 2 pad 1),
// forward.  The layer writes eight to thirty times more bytes than it reads, and its 3x3 windows
// are nine 2-byte elements per pixel: fetched from global memory they cost nine load instructions
// per 32 pixels, and the vector-memory instruction rate of a wave, not bandwidth, sets the pace.
// Here one loader wave copies each band's image rows (a few KiB, 1 KiB per load) into an LDS ring
// with LDS-writing 16-byte loads, seven compute waves take the band's pixels in groups of 32 (lane =
// pixel), gather the window from LDS (one channel: two dwords per window row; three: 2-byte reads), apply
// the weights with one or two MFMAs (K = 9*C0 padded to 16 or 32) whose accumulator starts at the
// bias, round to bf16, clamp, stage the 32 pixels in a private
// LDS strip and write them as 16-byte segments of the band's contiguous output span.  The images
// are addressed through the minibatch's gather list.
#pragma once
#include "conv_tile.hip.h"

struct Conv0Args {
  ImgAddr in;                 // input images [H][W][C0], gathered through in.idx
  bf16_t* out;                // output images [Ho][Wo][Cout], dense, image i at out + i*Ho*Wo*Cout
  const bf16_t* w;            // [Cout][9*C0]
  const float* bias;
  const bf16_t* zpage;        // 1 KiB of zeros
  uint32_t* bits;             // optional sign-bit words of the output (layout as in ConvTileArgs)
  int H, W, Ho, Wo, Cout;
  int TR, NB, ntiles;         // output rows per band, bands per image, nimg * NB
  FastDiv dv_wo;              // division by Wo
  // the blocks behind the tile_blocks tile blocks copy the samples' proprioception (bf16 in the rollout
  // buffer, gathered through in.idx) into columns [pcol0, pcol0 + P) of the feature matrix (gather_blocks = 0: none)
  int tile_blocks, gather_blocks, pB, P, pcol0;
  const bf16_t* proprio;
  bf16_t* feat;
  int64_t feat_ld;
};

template <int C0>
struct Conv0Shape {
  static constexpr int K = 9 * C0, KS = (K + 15) / 16, NBUF = 3, THREADS = 512, NCW = 7;
  static constexpr int MAXSEG = 2;
  static int image_bytes(int W, int TR) { return (2 * TR + 1) * W * C0 * 2; }
  static int lds_bytes(int W, int TR, int Cout) { return NBUF * image_bytes(W, TR) + 16 + NCW * 32 * (Cout + 8) * 2; }
};

template <int C0>
__global__ __launch_bounds__(512) void k_conv0_fwd_tile(Conv0Args a) {
  typedef Conv0Shape<C0> S;
  constexpr int K = S::K, KS = S::KS, NBUF = S::NBUF, NCW = S::NCW;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l32 = lane & 31, h = lane >> 5;
  const int W = a.W, TR = a.TR, Wo = a.Wo, Cout = a.Cout;
  const int RB = W * C0 * 2, nrows = 2 * TR + 1, image_bytes = nrows * RB;
  char* const zero16 = lds + NBUF * image_bytes;
  const int SP = Cout + 8;  // staging pitch (elements)
  if ((int)blockIdx.x >= a.tile_blocks) {
    const int64_t n = (int64_t)a.pB * a.P;
    for (int64_t i = (int64_t)((int)blockIdx.x - a.tile_blocks) * 512 + tid; i < n; i += (int64_t)a.gather_blocks * 512) {
      const int b = (int)(i / a.P), j = (int)(i - (int64_t)b * a.P);
      const int64_t s = a.in.idx ? a.in.idx[b] : b;
      a.feat[(int64_t)b * a.feat_ld + a.pcol0 + j] = a.proprio[s * a.P + j];
    }
    return;
  }
  const int nblk = a.tile_blocks;
  const int vb = xcd_block((int)blockIdx.x, nblk);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / nblk + 1 : 0;
  if (tid < 4) reinterpret_cast<uint32_t*>(zero16)[tid] = 0u;

  if (wave == 7) {
    // ------------------------------------------------------------------ loader
    // the band's rows follow each other in memory and in LDS: 1 KiB per load whatever the row length
    const int ni = (image_bytes + 1023) >> 10;
    auto issue = [&](int q) {
      const int t = vb + q * nblk;
      const int img = t / a.NB, band = t - img * a.NB;
      const int iy_lo = 2 * band * TR - 1;
      const char* src = reinterpret_cast<const char*>(a.in.ptr_uniform(img)) + (int64_t)iy_lo * RB;
      char* dst = lds + (q % NBUF) * image_bytes;
      for (int j = 0; j < ni; ++j) {
        const int o = j * 1024 + lane * 16, iy = iy_lo + o / RB;
        const bool inside = iy >= 0 && iy < a.H;
        const char* p = inside ? src + o : reinterpret_cast<const char*>(a.zpage) + lane * 16;
        if (o < image_bytes) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + j * 1024), 16, 0, 0);
      }
    };
    if (nq > 0) issue(0);
    if (nq > 1) issue(1);
    for (int q = 0; q < nq; ++q) {
      vm_wait_dyn(q + 1 < nq ? ni : 0);  // band q has landed
      __builtin_amdgcn_s_barrier();
      if (q + 2 < nq) issue(q + 2);
    }
    return;
  }

  // -------------------------------------------------------------------- compute waves
  bf16_t* const stage = reinterpret_cast<bf16_t*>(zero16 + 16) + wave * 32 * SP;
  const int NJ = (Cout + 31) / 32;
  // weights (MFMA first operand: row co = jn*32 + l32, 8 k at ks*16 + h*8) and bias per accumulator element
  bf16x8_t bw[2][KS];
  f32x16_t bs[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn) {
    const int co = jn * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint32_t t[4] = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = ks * 16 + h * 8 + j;
        const uint32_t x = (k < K && co < Cout) ? (uint32_t)a.w[co * K + k] : 0u;
        t[j >> 1] |= x << (16 * (j & 1));
      }
      bw[jn][ks] = __builtin_bit_cast(bf16x8_t, make_uint4(t[0], t[1], t[2], t[3]));
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) { const int c2 = jn * 32 + (e >> 2) * 8 + h * 4 + (e & 3); bs[jn][e] = c2 < Cout ? a.bias[c2] : 0.f; }
  }
  const int npix = TR * Wo, ngroups = (npix + 31) >> 5;
  const int cpr = Cout >> 3;  // 16-byte chunks per pixel
  const int cshift = (cpr & (cpr - 1)) == 0 ? 31 - __builtin_clz(cpr) : -1;  // log2 of it when it is a power of two
  const FastDiv dv_wo = a.dv_wo;
  const uint32_t negw = nonzero_weights(h);

  for (int q = 0; q < nq; ++q) {
    const int t = vb + q * nblk;
    const int img = t / a.NB, band = t - img * a.NB;
    const int plim = min(TR, a.Ho - band * TR) * Wo;  // pixels of the band that exist
    bf16_t* dst = a.out + ((int64_t)img * a.Ho + (int64_t)band * TR) * Wo * Cout;
    __builtin_amdgcn_s_barrier();  // band q is in LDS
    const char* im = lds + (q % NBUF) * image_bytes;
    for (int gi = wave; gi < ngroups; gi += NCW) {
      const int p = gi * 32 + l32, pc = p < npix ? p : 0;
      const int oyl = (int)dv_wo.div((uint32_t)pc), ox = pc - oyl * Wo;
      bf16x8_t av[KS];
      if constexpr (C0 == 1) {
        // three rows of the window as two dwords each: columns (2x-2, 2x-1) and (2x, 2x+1); W is even here (rows are
        // multiples of 16 bytes), so only the left edge needs a mask.  k = 3*u + v: half 0 takes taps 0..7, half 1 tap 8.
        const char* rowp = im + (2 * oyl) * RB + 4 * ox;
        const uint32_t lm = ox > 0 ? 0xffffffffu : 0u;
        uint32_t d0[3], d1[3];
#pragma unroll
        for (int u = 0; u < 3; ++u) {
          d1[u] = *reinterpret_cast<const uint32_t*>(rowp + u * RB);
          d0[u] = *reinterpret_cast<const uint32_t*>(rowp + u * RB + (ox > 0 ? -4 : 0)) & lm;
        }
        const uint32_t w0 = __builtin_amdgcn_alignbit(d1[0], d0[0], 16);       // (row 0: col -1, col 0)
        const uint32_t w1 = __builtin_amdgcn_perm(d0[1], d1[0], 0x07060302u);  // (row 0: col +1, row 1: col -1)
        const uint32_t w3 = __builtin_amdgcn_alignbit(d1[2], d0[2], 16);       // (row 2: col -1, col 0)
        av[0] = __builtin_bit_cast(bf16x8_t, h ? make_uint4(d1[2] >> 16, 0u, 0u, 0u) : make_uint4(w0, w1, d1[1], w3));
      } else {
        const char* pb = im + (2 * oyl) * RB + (2 * ox - 1) * C0 * 2;  // window corner (column -1 for ox = 0)
        const bool cok[3] = {ox > 0, true, 2 * ox + 1 < W};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
          uint32_t x4[4] = {0u, 0u, 0u, 0u};
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            // the two halves' k are compile-time; pick by h
            const int k0 = ks * 16 + j, k1 = ks * 16 + 8 + j;
            const int t0 = k0 / C0, c0 = k0 - t0 * C0, u0 = t0 / 3, v0 = t0 - 3 * u0;
            const int t1 = k1 / C0, c1 = k1 - t1 * C0, u1 = t1 / 3, v1 = t1 - 3 * u1;
            const bool in0 = k0 < K, in1 = k1 < K;
            const bool ok = h ? (in1 && cok[in1 ? v1 : 1]) : (in0 && cok[in0 ? v0 : 1]);
            const int off = h ? (in1 ? u1 * RB + (v1 * C0 + c1) * 2 : 0) : (in0 ? u0 * RB + (v0 * C0 + c0) * 2 : 0);
            const char* src = ok ? pb + off : zero16;
            x4[j >> 1] |= (uint32_t)*reinterpret_cast<const unsigned short*>(src) << (16 * (j & 1));
          }
          av[ks] = __builtin_bit_cast(bf16x8_t, make_uint4(x4[0], x4[1], x4[2], x4[3]));
        }
      }
      uint32_t pw[2] = {0u, 0u};
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) {
        if (jn < NJ) {
          f32x16_t acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw[jn][0], av[0], bs[jn], 0, 0, 0);  // the bias enters as the accumulator
#pragma unroll
          for (int ks = 1; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw[jn][ks], av[ks], acc, 0, 0, 0);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            // Cout is a multiple of 8: the eight columns of (jn, g) exist together, for both lane halves
            if (jn * 32 + g * 8 < Cout) {
              uint2 o;
              o.x = relu_pack2bf(acc[g * 4], acc[g * 4 + 1]);
              o.y = relu_pack2bf(acc[g * 4 + 2], acc[g * 4 + 3]);
              *reinterpret_cast<uint2*>(&stage[l32 * SP + jn * 32 + g * 8 + h * 4]) = o;
              pw[jn] |= nonzero4(o.x, o.y, negw) << (g * 8);
            }
          }
        }
      }
      if (a.bits) {
        const int wpp = (Cout + 31) >> 5;
        uint32_t* const bw0 = a.bits + ((int64_t)img * a.Ho * Wo + (int64_t)band * TR * Wo) * wpp;  // the band's words
#pragma unroll
        for (int jn = 0; jn < 2; ++jn) {
          const uint32_t word = or_with_lane_xor32(pw[jn]);
          if (h == 0 && jn < wpp && p < plim) bw0[(uint32_t)(p * wpp + jn)] = word;
        }
      }
      // the group's 32 pixels are contiguous in the output: chunk ch of the group is its bytes [16 ch, 16 ch + 16)
      bf16_t* const dst_g = dst + (int64_t)gi * 32 * Cout;
      const int plim_g = plim - gi * 32;
      for (int ch = lane; ch < 32 * cpr; ch += 64) {
        const int r = cshift >= 0 ? ch >> cshift : ch / cpr, cg = ch - r * cpr;
        if (r < plim_g)
          store_stream16(dst_g + (uint32_t)ch * 8u, *reinterpret_cast<const uint4*>(&stage[r * SP + cg * 8]));
      }
    }
  }
}
