// Input gradient of the second convolution (64 gradient channels -> 32 channels, 3x3 stride 2
// pad 1, transposed) fused with the weight gradient of the first convolution, whose input is the
// C0-channel observation image (C0 = 1 or 3).  The gradient of the first layer's output lives only
// in registers: it goes from the accumulators of the transposed convolution straight into the
// operands of the weight-gradient product.
//
// Quads (2x2 blocks of result pixels, see conv_dgrad_tile.hip.h) are the rows of the first product:
// D1[quad][ci] = sum over co of dY[pixel of the quad][co] * Wt[tap][ci][co], one accumulator per
// pixel class, with 16x16x32 MFMAs.  A lane of the result then holds, for ONE channel ci, four
// consecutive quads of each class: exactly the shape of the first operand of the second product
// G0[ci][k0] += sum over pixels of dXmasked[pixel][ci] * patch[pixel][k0], whose contraction index
// (32 per MFMA) runs over 4 lane groups x (2 horizontal classes x 4 quads).  The other operand,
// patch[pixel][k0], is gathered from the band's image rows in LDS by lane (k0 = lane % 16, same
// pixels): the eight window values of a lane are the same half of eight dwords, C0 dwords apart.  The ReLU mask of the first layer's output arrives as one 32-bit
// word per pixel (bit = channel); a lane keeps its value when bit ci of the pixel's word is set.
//
// A block has four or eight compute waves and four loader waves.  Compute wave w works on channels
// 16*(w&1) .. +15 (72 weight registers) and on quads 64*(w>>1) .. +63 of the tile (32 quads per
// compute wave); with eight, two compute waves share a SIMD and hide each other's LDS latency.  The
// loaders copy, per band, the dY rows (TQ+1), the image rows (4*TQ+1) and the mask words (2*TQ rows)
// into a ring of three LDS slots with LDS-writing 16-byte loads, 1 KiB per instruction; rows outside
// the images come from a page of zeros (64 KiB, so that a whole dY row outside the image is a scalar
// choice of base address), so no lane tests a row bound.  One barrier per tile: the
// loaders arrive when the band has landed, the compute waves when they are done with the previous
// one.
//
// The second product reads as little LDS as it can: the width in quads is a multiple of four, hence the
// four quads of a lane are neighbours in one row, their eight mask words are 32 contiguous bytes (two
// 16-byte reads) and the eight window values of a (tap, channel) are the low or high halves of eight
// dwords at a fixed pitch (read as dwords, two per instruction, halves picked with a byte permute; lanes
// without a patch column select zeros).  Every LDS offset of the
// second product is a per-lane constant plus an immediate.  Each block leaves one fp32 partial
// [32][9*C0+1] (last column: bias gradient, from a constant-one patch column).
//
// The instruction issue of the SIMDs is what bounds the kernel: at three to four vector instructions per
// MFMA the two kinds hardly overlap on a SIMD, whichever waves they come from (measured with a loop of one
// MFMA and K vector instructions), so every vector instruction counts.
// Hence: one per-lane offset per M-tile and kind of read (the second pixel row, the second half of the
// gradient channels and the window's dwords are reached through instruction offsets, with the row pitches
// known at compile time in the WC form); the bias column of that form reads a block of bf16 ones kept in
// the slot instead of being ORed into every window; lanes beyond the band read a tail of zeros behind the
// mask words, one mask row long, so that both pixel rows of a quad use one offset; loader waves whose
// address work per load is scalar.  For one-channel images the first product of M-tile m+1 and the second
// of M-tile m are written as ONE instruction stream in a fixed order (fused()).
#pragma once
#include "conv_dgrad_tile.hip.h"

typedef float f32x4_t __attribute__((ext_vector_type(4)));

template <int NCW>  // compute waves: 4 or 8
struct ConvDgradW0Shape {
  static constexpr int CI = 32, CO = 64, BQ = 32 * NCW, NBUF = 3, NLW = 4, THREADS = (NCW + NLW) * 64;
  static constexpr int MAXSEG = 24, MAXI = 4, MAXM = 2;  // 1 KiB parts of a dY row; loads per loader wave and band: image rows, mask words
  static int dyimg_bytes(int Wo, int TQ) { return (TQ + 1) * (Wo + 1) * 128; }
  static int img0_bytes(int W0, int C0, int TQ) { return (4 * TQ + 1) * W0 * C0 * 2; }
  static int mask_bytes(int W, int TQ) { return 2 * TQ * W * 4; }
  // ones: the slot ends with the block of bf16 ones of the forms whose width is known at compile time (one-channel images)
  static int slot_bytes(int W, int Wo, int W0, int C0, int TQ, bool ones) {
    return dyimg_bytes(Wo, TQ) + img0_bytes(W0, C0, TQ) + 16 + mask_bytes(W, TQ) + W * 4 + 32 + (ones ? 4 * W0 * C0 + 32 : 0);
  }
  static int ring_bytes(int W, int Wo, int W0, int C0, int TQ, bool ones) {
    const int r = NBUF * slot_bytes(W, Wo, W0, C0, TQ, ones);
    return r > NCW * 2048 ? r : NCW * 2048;  // the final sums of the wave pairs reuse the ring
  }
  static int lds_bytes(int W, int Wo, int W0, int C0, int TQ, bool ones) { return ring_bytes(W, Wo, W0, C0, TQ, ones); }
  // dY loads of the busiest loader wave per band: whole rows in turn, or a quarter of the parts of every row
  static int dy_loads(int Wo, int TQ, int split) {
    const int segs = (Wo * 128 + 1023) / 1024;
    return split ? (TQ + 1) * ((segs + NLW - 1) / NLW) : ((TQ + 1 + NLW - 1) / NLW) * segs;
  }
  static int seg_split(int Wo, int TQ) { return dy_loads(Wo, TQ, 1) < dy_loads(Wo, TQ, 0) ? 1 : 0; }
  static bool loads_fit(int W, int Wo, int W0, int C0, int TQ) {
    const int segs = (Wo * 128 + 1023) / 1024;
    return segs <= MAXSEG && dy_loads(Wo, TQ, seg_split(Wo, TQ)) + MAXI + MAXM <= 63 && (img0_bytes(W0, C0, TQ) + 1023) / 1024 <= MAXI * NLW &&
           (mask_bytes(W, TQ) + 1023) / 1024 <= MAXM * NLW;
  }
};

// Requires (checked by the host): W % 8 == 0 (Wo % 4 == 0), (W0 * C0 * 2) % 16 == 0, Wo == W / 2 <= BQ, TQ * Wo <= BQ.
// WC: the width W of the result known at compile time (row pitches become instruction offsets), or 0: taken from a.W.
template <int C0, int NCW, int WC>
__global__ __launch_bounds__((NCW + 4) * 64) void k_conv_dgrad_wgrad0_tile(ConvDgradArgs a) {
  typedef ConvDgradW0Shape<NCW> S;
  constexpr int BQ = S::BQ;
  constexpr int NBUF = S::NBUF, K0 = 9 * C0, NV = K0 + 1, NT = (NV + 15) / 16;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int W = WC ? WC : a.W, Wo = WC ? WC / 2 : a.Wo, TQ = a.TQ;
  const int RP = (Wo + 1) * 128, dyimg_bytes = (TQ + 1) * RP;  // dY image: row pitch, bytes
  const int RB0 = (WC ? 2 * WC : a.W0) * C0 * 2, img0_bytes = (4 * TQ + 1) * RB0;
  const int MRB = W * 4, mask_bytes = 2 * TQ * MRB;
  // slot: dY image | image rows | 16 zero bytes | mask words | one row of mask words + 32 bytes of zeros |
  // one-channel images: 32 bytes of bf16 ones, and 32 more two image rows further (the window of the bias column)
  const int OFF_IMG = dyimg_bytes, OFF_MSK = OFF_IMG + img0_bytes + 16, OFF_Z = OFF_MSK + mask_bytes, OFF_ONES = OFF_Z + MRB + 32;
  constexpr bool ONES = C0 == 1 && WC != 0;  // the bias column reads a block of ones (costs 2 image rows of LDS per slot) instead of being ORed in
  const int SLOT = OFF_ONES + (ONES ? 2 * RB0 + 32 : 0);
  const int vb = xcd_block((int)blockIdx.x, (int)gridDim.x);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / (int)gridDim.x + 1 : 0;

  // ---- once: the zero pads no load ever writes
  for (int i = tid; i < NBUF * (TQ + 1) * 8; i += S::THREADS) {
    const int chunk = i & 7, row = i >> 3, s = row / (TQ + 1), rr = row - s * (TQ + 1);
    *reinterpret_cast<uint4*>(lds + s * SLOT + rr * RP + Wo * 128 + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }
  {
    const int nz = 1 + (MRB + 32) / 16;  // 16-byte pieces of zeros per slot: one behind the image rows, the tail behind the mask words
    for (int i = tid; i < NBUF * nz; i += S::THREADS) {
      const int s = i / nz, k = i - nz * s, off = k == 0 ? OFF_IMG + img0_bytes : OFF_Z + (k - 1) * 16;
      *reinterpret_cast<uint4*>(lds + s * SLOT + off) = make_uint4(0u, 0u, 0u, 0u);
    }
    if (ONES && tid < NBUF * 4) {
      const int s = tid >> 2, k = tid & 3;
      *reinterpret_cast<uint4*>(lds + s * SLOT + OFF_ONES + (k >> 1) * 2 * RB0 + (k & 1) * 16) = make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u);
    }
  }

  if (wave >= NCW) {
    // ------------------------------------------------------------------ loaders: piece i of a band belongs to loader i % 4
    const int lw = wave - NCW;
    const int rowbytes = Wo * 128, segs = (rowbytes + 1023) >> 10;
    const int n_im = (img0_bytes + 1023) >> 10, n_mk = (mask_bytes + 1023) >> 10;
    // piece j of a kind (rows of the dY image, 1 KiB pieces of the image rows, of the mask words) belongs to loader j % 4
    auto mine = [&](int n) { return n > lw ? (n - lw + S::NLW - 1) / S::NLW : 0; };
    const int mysegs = segs > lw ? (segs - lw + S::NLW - 1) / S::NLW : 0;  // parts lw, lw + 4, ... of a row
    const int nd = a.seg_split ? (TQ + 1) * mysegs : mine(TQ + 1) * segs, nm_i = mine(n_im), nm_m = mine(n_mk);
    const int ni = nd + nm_i + nm_m;  // this wave's loads per band
    const char* const zp = reinterpret_cast<const char*>(a.zpage) + lane * 16;
    // dY rows are copied in parts of 1 KiB, a loader taking whole rows in turn or (few rows of many parts) its
    // share of the parts of every row: what a lane adds to the row's address depends on the part alone
    // (the 16-byte chunks of a pixel are permuted, dy_swz_bits, through the source address), and a row is inside
    // the image or not for the whole wave, so that the choice between the image and the page of zeros (a.zpage:
    // 64 KiB) and every other address part is scalar work: one vector instruction per load.  The lanes beyond
    // the end of a row whose last part is shorter than 1 KiB sit out.
    constexpr int MAXSEG = S::MAXSEG, MAXI = S::MAXI, MAXM = S::MAXM;
    constexpr int MYSEG = MAXSEG / S::NLW;
    int lo[MAXSEG], mylo[MYSEG], igo[MAXI], irow[MAXI], mgo[MAXM], mrow[MAXM];
#pragma unroll
    for (int sg = 0; sg < MAXSEG; ++sg) {
      const uint32_t phys = sg * 1024 + lane * 16;
      lo[sg] = (int)(phys ^ dy_swz_bits(phys));
    }
#pragma unroll
    for (int j = 0; j < MYSEG; ++j) {
      const uint32_t phys = (lw + S::NLW * j) * 1024 + lane * 16;
      mylo[j] = (int)(phys ^ dy_swz_bits(phys));
    }
    const int tail = rowbytes - (segs - 1) * 1024;
    const bool in_tail = lane * 16 < tail;
    const char* const zbase = reinterpret_cast<const char*>(a.zpage);
#pragma unroll
    for (int k = 0; k < MAXI; ++k) {
      const int o = (lw + S::NLW * k) * 1024 + lane * 16;
      irow[k] = (int)a.dv_rb0.div((uint32_t)o); igo[k] = o < img0_bytes ? o : -1;
    }
#pragma unroll
    for (int k = 0; k < MAXM; ++k) {
      const int o = (lw + S::NLW * k) * 1024 + lane * 16;
      mrow[k] = (int)a.dv_mrow.div((uint32_t)o); mgo[k] = o < mask_bytes ? o : -1;
    }
    // tiles of this block in order: (img, band) advances by gridDim.x tiles without a division
    const int step_img = (int)gridDim.x / a.NB, step_band = (int)gridDim.x - step_img * a.NB;
    int n_img = vb / a.NB, n_band = vb - n_img * a.NB;
    struct Band { const char* base[3]; int r0[3]; };
    // base addresses and first rows of the next band to issue; formed one band ahead, so that the
    // scalar load of the gather index is not waited for
    auto prep = [&]() __attribute__((always_inline)) {
      Band b;
      const int img = n_img, band = n_band;
      b.r0[0] = band * TQ; b.r0[1] = 4 * band * TQ - 1; b.r0[2] = 2 * band * TQ;
      b.base[0] = reinterpret_cast<const char*>(a.dy.ptr_uniform(img)) + (int64_t)b.r0[0] * rowbytes;
      b.base[1] = reinterpret_cast<const char*>(a.img0.ptr_uniform(img)) + (int64_t)b.r0[1] * RB0;
      b.base[2] = reinterpret_cast<const char*>(a.xbits + ((int64_t)img * a.H + b.r0[2]) * W);
      n_img += step_img; n_band += step_band;
      if (n_band >= a.NB) { n_band -= a.NB; ++n_img; }
      return b;
    };
    Band nxt = prep();
    auto issue = [&](int q) __attribute__((always_inline)) {  // called for q = 0, 1, 2, ... in order
      const Band b = nxt;
      if (q + 1 < nq) nxt = prep();
      char* const slot = lds + (q % NBUF) * SLOT;
      const int nrows = a.Ho - b.r0[0];  // rows of the image from the band's first one on
      if (a.seg_split) {
        for (int row = 0; row <= TQ; ++row) {
          const char* const base = row < nrows ? b.base[0] + row * rowbytes : zbase;  // rows outside the image: zeros
          char* const dst = slot + row * RP;
#pragma unroll
          for (int j = 0; j < MYSEG; ++j) {
            const int sg = lw + S::NLW * j;
            if (sg < segs) {
              const char* p = base + mylo[j];
              if (sg == segs - 1 && tail < 1024) {
                if (in_tail) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + sg * 1024), 16, 0, LOAD_NT);
              } else {
                __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + sg * 1024), 16, 0, LOAD_NT);
              }
            }
          }
        }
      } else {
        for (int row = lw; row <= TQ; row += S::NLW) {
          const char* const base = row < nrows ? b.base[0] + row * rowbytes : zbase;  // rows outside the image: zeros
          char* const dst = slot + row * RP;
#pragma unroll
          for (int sg = 0; sg < MAXSEG; ++sg)
            if (sg < segs) {
              const char* p = base + lo[sg];
              if (sg == segs - 1 && tail < 1024) {
                if (in_tail) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + sg * 1024), 16, 0, LOAD_NT);
              } else {
                __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + sg * 1024), 16, 0, LOAD_NT);
              }
            }
        }
      }
#pragma unroll
      for (int k = 0; k < MAXI; ++k)
        if (k < nm_i) {
          const char* p = ((uint32_t)(b.r0[1] + irow[k]) < (uint32_t)a.H0) ? b.base[1] + igo[k] : zp;
          if (igo[k] >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(slot + OFF_IMG + (lw + S::NLW * k) * 1024), 16, 0, 0);
        }
#pragma unroll
      for (int k = 0; k < MAXM; ++k)
        if (k < nm_m) {
          const char* p = (b.r0[2] + mrow[k] < a.H) ? b.base[2] + mgo[k] : zp;
          if (mgo[k] >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(slot + OFF_MSK + (lw + S::NLW * k) * 1024), 16, 0, LOAD_NT);
        }
    };
    // bands 0 and 1 are issued before the first wait: the loop starts two bands early
    for (int q = -2; q < nq; ++q) {
      if (q >= 0) {
        vm_wait_dyn(q + 1 < nq ? ni : 0);  // band q has landed
        __builtin_amdgcn_s_barrier();      // A(q); the compute waves have left band q - 1
      }
      if (q + 2 < nq) issue(q + 2);
    }
    __builtin_amdgcn_s_barrier();        // C
    __builtin_amdgcn_s_barrier();        // D
    return;
  }

  // -------------------------------------------------------------------- compute waves
  const int l16 = lane & 15, r = lane >> 4, ch = wave & 1, gp = wave >> 1;
  // weights, second operand of the first product: lane (column ci = ch*16 + l16, 8 co at ks*32 + r*8) of tap s
  bf16x8_t wr[9][2];
#pragma unroll
  for (int s = 0; s < 9; ++s)
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      wr[s][ks] = *reinterpret_cast<const bf16x8_t*>(a.wt + ((int64_t)s * 32 + ch * 16 + l16) * 64 + ks * 32 + r * 8);
  // first operand: lane (row = quad gp*64 + m*16 + l16, 8 co at ks*32 + r*8); xa[m][dxo]: this lane's chunk of the quad's
  // pixel (+ dxo) in a dY image for ks = 0; the chunk for ks = 1 is at xa ^ 64 (rows and pixels are multiples of 128 bytes)
  int xa[4][2];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int qi = gp * 64 + m * 16 + l16;
    const bool valid = qi < TQ * Wo;  // lanes beyond the band work on quad 0; their results meet zero mask words
    const int al = valid ? qi / Wo : 0, b = valid ? qi - al * Wo : 0;
#pragma unroll
    for (int dxo = 0; dxo < 2; ++dxo) xa[m][dxo] = al * RP + (b + dxo) * 128 + (int)((uint32_t)(r * 16) ^ dy_swz_bits((uint32_t)((b + dxo) * 128)));
    // (opaque from here on: a sum the compiler can see through is split again into parts that cost an addition per read)
    asm volatile("" : "+v"(xa[m][0]), "+v"(xa[m][1]));
  }
  const int cibit = ch * 16 + l16;  // this lane's channel as a result column: its bit in a mask word
  // second product, second operand: lane (column k0 = nt*16 + l16, pixels of lane group r)
  int toffl[NT];
  uint32_t lnv0[NT], bconst[NT], hsel[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int k0 = nt * 16 + l16;
    const bool real = k0 < K0;
    const int tap = real ? k0 / C0 : 1, cch = real ? k0 - tap * C0 : 0, u = tap / 3, v = tap - 3 * u;
    // window corner is (row - 1, column - 1)
    // The window value of (tap column v, channel cch) at pixel column x is element C0*(x + v - 1) + cch of the row; x
    // advances by 2 per window value, an even number of elements: all eight values of a lane are the same half of
    // dwords that are C0 dwords apart.  e0: the element for x = 0 (it may lie left of the image: -C0 .. -1).
    const int e0 = C0 * (v - 1) + cch;
    toffl[nt] = u * RB0 + 4 * (e0 >> 1);
    hsel[nt] = (!real && !(ONES && k0 == K0)) ? 0x0c0c0c0cu : ((e0 & 1) ? 0x07060302u : 0x05040100u);  // selector bytes 0x0c give zero
    lnv0[nt] = v != 0 ? 0xfu : 0u;
    bconst[nt] = k0 == K0 ? 0x3F803F80u : 0u;  // the bias column: 1.0
  }
  // this lane's four quads of M-tile m are q0 .. q0 + 3, q0 = gp*64 + m*16 + r*4, neighbours in one quad row;
  // groups beyond the band read the zero words behind the mask (both pixel rows: the second is one row of mask
  // words further) and any real window.  kpb[nt], bit m: the first window value of M-tile m is kept (it is dropped
  // where it is the column left of the image: lanes of column 0 with a tap of the window's first column).
  int mo[4], go[4];
  uint32_t kpb[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) kpb[nt] = lnv0[nt];
#pragma unroll
  for (int m = 0; m < 4; ++m) {
    const int q0 = gp * 64 + m * 16 + r * 4;
    const bool valid = q0 < TQ * Wo;
    const int al = valid ? q0 / Wo : 0, b = valid ? q0 - al * Wo : 0;
    mo[m] = valid ? OFF_MSK + ((2 * al) * W + 2 * b) * 4 : OFF_Z;
    go[m] = OFF_IMG + 4 * al * RB0 + 8 * b * C0 + (NT == 1 ? toffl[0] : 0);
    if (ONES && l16 == K0) go[m] = OFF_ONES;  // the bias column reads ones
    if (!(valid && b == 0)) {
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) kpb[nt] |= 1u << m;
    }
    asm volatile("" : "+v"(mo[m]), "+v"(go[m]));
  }
  f32x4_t accw[NT];
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) accw[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};

  auto dgrad = [&](const char* slot, int m, f32x4_t (&acc)[4]) __attribute__((always_inline)) {
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int pi = 0; pi < 4; ++pi) {
      const int dyo = pi >> 1, dxo = pi & 1;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8_t x = *reinterpret_cast<const bf16x8_t*>(slot + dyo * RP + (xa[m][dxo] ^ (ks * 64)));
        // class (py, px) takes tap row py ? (dyo ? 0 : 2) : 1 from row offset dyo (even rows only from dyo = 0), same for columns
        if (pi == 0) {
          acc[0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[1 * 3 + 1][ks], acc[0], 0, 0, 0);
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[1 * 3 + 2][ks], acc[1], 0, 0, 0);
          acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[2 * 3 + 1][ks], acc[2], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[2 * 3 + 2][ks], acc[3], 0, 0, 0);
        } else if (pi == 1) {
          acc[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[1 * 3 + 0][ks], acc[1], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[2 * 3 + 0][ks], acc[3], 0, 0, 0);
        } else if (pi == 2) {
          acc[2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[0 * 3 + 1][ks], acc[2], 0, 0, 0);
          acc[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[0 * 3 + 2][ks], acc[3], 0, 0, 0);
        } else {
          acc[3] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x, wr[0 * 3 + 0][ks], acc[3], 0, 0, 0);
        }
      }
    }
  };
  // acc[c][i] = dX[quad gp*64 + m*16 + r*4 + i, class c][ci]
  auto wgrad = [&](const char* slot, int m, const f32x4_t (&acc)[4]) __attribute__((always_inline)) {
#pragma unroll
    for (int py = 0; py < 2; ++py) {
      // the mask words of the four quads' eight pixels in this row: word 2*i + px
      const uint4 wa = *reinterpret_cast<const uint4*>(slot + mo[m] + py * MRB), wb = *reinterpret_cast<const uint4*>(slot + mo[m] + py * MRB + 16);
      const uint32_t w[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
      float v0[4], v1[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int k0 = __builtin_amdgcn_sbfe((int)w[2 * i], (uint32_t)cibit, 1u), k1 = __builtin_amdgcn_sbfe((int)w[2 * i + 1], (uint32_t)cibit, 1u);
        const float d0 = acc[py * 2][i], d1 = acc[py * 2 + 1][i];
        v0[i] = __int_as_float(__float_as_int(d0) & k0);
        v1[i] = __int_as_float(__float_as_int(d1) & k1);
      }
      const bf16x8_t av = __builtin_bit_cast(bf16x8_t, make_uint4(pack2bf(v0[0], v0[1]), pack2bf(v0[2], v0[3]), pack2bf(v1[0], v1[1]), pack2bf(v1[2], v1[3])));
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) {
        const char* p = slot + go[m] + (NT == 1 ? 0 : toffl[nt]) + 2 * py * RB0;
        const uint32_t km = (uint32_t)__builtin_amdgcn_sbfe((int)kpb[nt], (uint32_t)m, 1u);
        uint4 bq;
        uint32_t d[8];  // window value k = 2*i + px: dword C0*k from the lane's first
#pragma unroll
        for (int k = 0; k < 8; ++k) d[k] = *reinterpret_cast<const uint32_t*>(p + 4 * C0 * k);
        d[0] &= km;
        bq = make_uint4(__builtin_amdgcn_perm(d[2], d[0], hsel[nt]), __builtin_amdgcn_perm(d[6], d[4], hsel[nt]),
                        __builtin_amdgcn_perm(d[3], d[1], hsel[nt]), __builtin_amdgcn_perm(d[7], d[5], hsel[nt]));
        if constexpr (!ONES) { bq.x |= bconst[nt]; bq.y |= bconst[nt]; bq.z |= bconst[nt]; bq.w |= bconst[nt]; }
        accw[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, __builtin_bit_cast(bf16x8_t, bq), accw[nt], 0, 0, 0);
      }
    }
  };

  // The first product of M-tile m + 1 and the second product of M-tile m as ONE instruction
  // stream in a fixed order.  Left to itself the scheduler puts the 18 MFMAs of the first product in a row and the
  // ~70 vector instructions of the second behind them, with the LDS reads of each right in front of their first
  // use.  Here every MFMA of the first product is followed by four or five vector instructions of the
  // second (mask bits, masking, conversion, window halves), and every LDS read is issued three to eight MFMAs
  // before its first use.  The order of the additions into each accumulator is the one of dgrad() / wgrad().
  auto fused = [&](const char* slot, int m, const f32x4_t (&cur)[4], f32x4_t (&nxt)[4]) __attribute__((always_inline)) {
    auto xr = [&](int xi) __attribute__((always_inline)) {
      const int pi = xi >> 1, ks = xi & 1, dyo = pi >> 1, dxo = pi & 1;
      return *reinterpret_cast<const bf16x8_t*>(slot + dyo * RP + (xa[m + 1][dxo] ^ (ks * 64)));
    };
    bf16x8_t x[8];
    uint32_t w[8], v[8], d[8];
    uint4 bq;
    auto masks = [&](int py, int half) __attribute__((always_inline)) {  // words 4*half .. 4*half + 3 of the row
      const uint4 wa = *reinterpret_cast<const uint4*>(slot + mo[m] + py * MRB + 16 * half);
      w[4 * half + 0] = wa.x; w[4 * half + 1] = wa.y; w[4 * half + 2] = wa.z; w[4 * half + 3] = wa.w;
    };
    auto window = [&](int py, int nt = 0) __attribute__((always_inline)) {
      const char* p = slot + go[m] + (NT == 1 ? 0 : toffl[nt]) + 2 * py * RB0;
#pragma unroll
      for (int k = 0; k < 8; ++k) d[k] = *reinterpret_cast<const uint32_t*>(p + 4 * C0 * k);
    };
    // word e = 2*i + px belongs to value i of class (py, px); the operand takes the values of px = 0 first
    auto keep2 = [&](int py, int e0) __attribute__((always_inline)) {
#pragma unroll
      for (int e = e0; e < e0 + 2; ++e)
        v[e] = (uint32_t)__float_as_int(cur[py * 2 + (e & 1)][e >> 1]) & (uint32_t)__builtin_amdgcn_sbfe((int)w[e], (uint32_t)cibit, 1u);
    };
    uint4 aq;
    auto conv_lo = [&]() __attribute__((always_inline)) {
      aq.x = pack2bf(__int_as_float((int)v[0]), __int_as_float((int)v[2])); aq.z = pack2bf(__int_as_float((int)v[1]), __int_as_float((int)v[3]));
    };
    auto conv_hi = [&]() __attribute__((always_inline)) {
      aq.y = pack2bf(__int_as_float((int)v[4]), __int_as_float((int)v[6])); aq.w = pack2bf(__int_as_float((int)v[5]), __int_as_float((int)v[7]));
    };
    auto halves = [&](int nt = 0) __attribute__((always_inline)) {
      d[0] &= (uint32_t)__builtin_amdgcn_sbfe((int)kpb[nt], (uint32_t)m, 1u);
      bq = make_uint4(__builtin_amdgcn_perm(d[2], d[0], hsel[nt]), __builtin_amdgcn_perm(d[6], d[4], hsel[nt]),
                      __builtin_amdgcn_perm(d[3], d[1], hsel[nt]), __builtin_amdgcn_perm(d[7], d[5], hsel[nt]));
    };
    auto ones = [&](int nt = 0) __attribute__((always_inline)) {
      if constexpr (!ONES) { bq.x |= bconst[nt]; bq.y |= bconst[nt]; bq.z |= bconst[nt]; bq.w |= bconst[nt]; }
    };
    auto second = [&](int nt = 0) __attribute__((always_inline)) {
      accw[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, aq), __builtin_bit_cast(bf16x8_t, bq), accw[nt], 0, 0, 0);
    };
#define DW0_MF(c, xi, s, ks) nxt[c] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(x[xi], wr[s][ks], nxt[c], 0, 0, 0)
#define DW0_FENCE() __builtin_amdgcn_sched_barrier(0)
#pragma unroll
    for (int c = 0; c < 4; ++c) nxt[c] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    if constexpr (NT == 2) {
      // two 16-column tiles of the second product per pixel row (the bias column is in the second)
      masks(0, 0); x[0] = xr(0); DW0_FENCE();
      DW0_MF(0, 0, 4, 0); keep2(0, 0); masks(0, 1); DW0_FENCE();
      DW0_MF(1, 0, 5, 0); keep2(0, 2); conv_lo(); x[1] = xr(1); DW0_FENCE();
      DW0_MF(2, 0, 7, 0); keep2(0, 4); window(0, 0); DW0_FENCE();
      DW0_MF(3, 0, 8, 0); keep2(0, 6); conv_hi(); DW0_FENCE();
      DW0_MF(0, 1, 4, 1); masks(1, 0); DW0_FENCE();
      DW0_MF(1, 1, 5, 1); halves(0); DW0_FENCE();
      DW0_MF(2, 1, 7, 1); window(0, 1); x[2] = xr(2); DW0_FENCE();
      DW0_MF(3, 1, 8, 1); masks(1, 1); DW0_FENCE();
      second(0); x[3] = xr(3); DW0_FENCE();
      DW0_MF(1, 2, 3, 0); halves(1); ones(1); DW0_FENCE();
      second(1); x[4] = xr(4); DW0_FENCE();
      DW0_MF(3, 2, 6, 0); keep2(1, 0); DW0_FENCE();
      DW0_MF(1, 3, 3, 1); keep2(1, 2); conv_lo(); DW0_FENCE();
      DW0_MF(3, 3, 6, 1); keep2(1, 4); window(1, 0); x[5] = xr(5); DW0_FENCE();
      DW0_MF(2, 4, 1, 0); keep2(1, 6); conv_hi(); DW0_FENCE();
      DW0_MF(3, 4, 2, 0); x[6] = xr(6); DW0_FENCE();
      DW0_MF(2, 5, 1, 1); halves(0); DW0_FENCE();
      DW0_MF(3, 5, 2, 1); window(1, 1); x[7] = xr(7); DW0_FENCE();
      second(0); DW0_FENCE();
      DW0_MF(3, 6, 0, 0); DW0_FENCE();
      DW0_MF(3, 7, 0, 1); halves(1); ones(1); DW0_FENCE();
      second(1); DW0_FENCE();
    } else {
    masks(0, 0); x[0] = xr(0); DW0_FENCE();
    DW0_MF(0, 0, 4, 0); keep2(0, 0); masks(0, 1); DW0_FENCE();
    DW0_MF(1, 0, 5, 0); keep2(0, 2); conv_lo(); x[1] = xr(1); DW0_FENCE();
    DW0_MF(2, 0, 7, 0); keep2(0, 4); window(0); DW0_FENCE();
    DW0_MF(3, 0, 8, 0); keep2(0, 6); conv_hi(); DW0_FENCE();
    DW0_MF(0, 1, 4, 1); masks(1, 0); DW0_FENCE();
    DW0_MF(1, 1, 5, 1); halves(); DW0_FENCE();
    DW0_MF(2, 1, 7, 1); ones(); x[2] = xr(2); DW0_FENCE();
    DW0_MF(3, 1, 8, 1); masks(1, 1); DW0_FENCE();
    second(); x[3] = xr(3); DW0_FENCE();
    DW0_MF(1, 2, 3, 0); keep2(1, 0); DW0_FENCE();
    DW0_MF(3, 2, 6, 0); keep2(1, 2); conv_lo(); DW0_FENCE();
    DW0_MF(1, 3, 3, 1); keep2(1, 4); window(1); x[4] = xr(4); DW0_FENCE();
    DW0_MF(3, 3, 6, 1); keep2(1, 6); conv_hi(); DW0_FENCE();
    DW0_MF(2, 4, 1, 0); x[5] = xr(5); DW0_FENCE();
    DW0_MF(3, 4, 2, 0); halves(); DW0_FENCE();
    DW0_MF(2, 5, 1, 1); ones(); x[6] = xr(6); DW0_FENCE();
    second(); x[7] = xr(7); DW0_FENCE();
    DW0_MF(3, 5, 2, 1); DW0_FENCE();
    DW0_MF(3, 6, 0, 0);
    DW0_MF(3, 7, 0, 1); DW0_FENCE();
    }
#undef DW0_MF
#undef DW0_FENCE
  };

  for (int q = 0; q < nq; ++q) {
    __builtin_amdgcn_s_barrier();  // A(q): band q is in LDS (the first one also orders the zero pads)
    const char* slot = lds + (q % NBUF) * SLOT;
    // the first product of M-tile m + 1 is independent of the second product of M-tile m
    f32x4_t acc[2][4];
    dgrad(slot, 0, acc[0]);
#pragma unroll
    for (int m = 0; m < 4; ++m) {
      if constexpr (NT <= 2) {
        if (m + 1 < 4) fused(slot, m, acc[m & 1], acc[(m + 1) & 1]);
        else wgrad(slot, m, acc[m & 1]);
      } else {
        if (m + 1 < 4) dgrad(slot, m + 1, acc[(m + 1) & 1]);
        wgrad(slot, m, acc[m & 1]);
      }
    }
  }
  __builtin_amdgcn_s_barrier();    // C: nobody reads the ring any more
  float* const red = reinterpret_cast<float*>(lds);
  // accw[nt][i] = G0[ci = ch*16 + r*4 + i][k0 = nt*16 + l16], summed over this wave's quads
#pragma unroll
  for (int nt = 0; nt < NT; ++nt)
#pragma unroll
    for (int i = 0; i < 4; ++i) red[(gp * 32 + ch * 16 + r * 4 + i) * 32 + nt * 16 + l16] = accw[nt][i];
  __builtin_amdgcn_s_barrier();    // D
  float* P = a.partial0 + (int64_t)blockIdx.x * 32 * NV;
  for (int i = tid; i < 32 * NV; i += NCW * 64) {
    const int ci = i / NV, k = i - ci * NV;
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < NCW / 2; ++g) sum += red[g * 1024 + ci * 32 + k];
    P[i] = sum;
  }
}
