// 3x3 stride-2 pad-1 convolution forward for 32 or 64 input channels, organised around what is
// scarce on the CU for this shape: bytes in flight per CU and vector-ALU issue slots, not MFMA
// cycles.
//
//  * Persistent blocks walk over tiles = (image, band of TR output rows).  The band's input rows
//    (2*TR+1 of them, one contiguous span of the channel-last image) are copied as they are into
//    an LDS image; the im2col gather happens at LDS-read time, where a tap is a constant byte
//    offset from the lane's window corner.  Every input byte crosses the memory path once per block.
//  * The copy is done by four extra waves with loads that write LDS directly (global_load_lds_dwordx4,
//    lane l's 16 bytes land at the instruction's LDS base + 16*l), into a ring of nbuf images
//    (three for the large layers, as many as fit up to MAXBUF for small ones, whose bands are too few bytes to
//    cover the memory latency two at a time): nbuf - 1 bands are in flight while one is computed.  (One wave alone sustains only about one such
//    load per 190 cycles.)  A loader's own vmcnt counts only these loads, so "band q has landed" is an exact wait; one barrier per tile hands the image over and
//    returns the ring slot consumed one tile earlier.
//  * Each image row has a zero pixel to its left and right (written once), rows outside the image
//    are copied from a page of zeros: the padding needs no test at read time.
//  * Pixels are stored unpadded; the 16-byte chunks of a pixel are permuted by its slot index
//    (chunk ^ f(slot)), applied by the loader through the global address, so that the stride-2
//    operand reads spread over the banks (two lanes per bank group instead of eight or sixteen).
//  * A compute wave keeps its slice of the weight matrix (9*CIN deep, 64 or 32 columns: 144
//    registers) in registers for the whole kernel, and its lanes' pixel -> LDS offset is the same
//    for every tile.
//  * Each compute wave stages its 32 output pixels in a private LDS strip and writes them as
//    16-byte row segments; a band's outputs are one contiguous span of the output image.
#pragma once
#include "common.hip.h"
#include "gemm_dma.hip.h"

struct ConvTileArgs {
  ImgAddr in;                 // input images [H][W][CIN], dense
  bf16_t* out;                // output images [Ho][Wo][Cout] at out + b*out_stride_b + v*out_stride_v
  int64_t out_stride_b, out_stride_v;
  const bf16_t* w;            // [Cout][9*CIN], k = (u*3+v)*CIN + ci
  const float* bias;          // [Cout]
  const bf16_t* zpage;        // 1 KiB of zeros
  uint32_t* bits;             // optional: one bit per output element (stored value > 0), word w of pixel p of image i at
                              // bits[(i*Ho*Wo + p) * ceil(Cout/32) + w]; read by the transposed convolution as ReLU mask
  int V, H, W, Ho, Wo, Cout;
  int TR, NB, ntiles;         // output rows per band, bands per image, nimg * NB
  int nbuf;                   // ring images (3 .. MAXBUF)
};

// bf16 pair of (max(lo, 0), max(hi, 0)): rounded first, then clamped as 16-bit integers (a negative bf16 is a
// negative int16, and rounding keeps the sign, so the order of rounding and clamping does not matter)
__device__ __forceinline__ uint32_t relu_pack2bf(float lo, float hi) {
  typedef short s16x2_t __attribute__((ext_vector_type(2)));
  const s16x2_t z = {0, 0};
  return __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(s16x2_t, pack2bf(lo, hi)), z));
}
// Which of the four non-negative bf16 of the pairs (x, y) are non-zero, as bits 0..3 times the weight the caller's
// negw encodes (nonzero_weights: 1, or 16 for the upper nibble of a byte), added to acc.  A half is at most 0x7fff, so
// x + 0x7fff7fff carries "non-zero" into each half's top bit without a carry between the halves; the byte permute's
// sign selectors spread the four top bits to bytes 0x00 / 0xff (= -1), and the signed 4-byte dot product with the
// weights -1, -2, -4, -8 (or -16 .. -128) sums them.
// x of this lane OR x of the lane 32 away (one half-wave swap instead of a permute through LDS): either returned half
// holds the own value and the other the partner's, so the OR of both is independent of which is which
__device__ __forceinline__ uint32_t or_with_lane_xor32(uint32_t x) {
  const auto r = __builtin_amdgcn_permlane32_swap(x, x, false, false);
  return r[0] | r[1];
}
__device__ __forceinline__ uint32_t nonzero_weights(int upper) { return upper ? 0x80c0e0f0u : 0xf8fcfeffu; }
__device__ __forceinline__ uint32_t nonzero4(uint32_t x, uint32_t y, uint32_t negw) {
  const uint32_t tx = x + 0x7fff7fffu, ty = y + 0x7fff7fffu;
  const uint32_t s = __builtin_amdgcn_perm(ty, tx, 0x0b0a0908u);
  return (uint32_t)__builtin_amdgcn_sdot4((int)s, (int)negw, 0, false);
}

template <int CIN, int WIDE = 0>
struct ConvTileShape {
  static_assert(!WIDE || CIN == 64, "the wide form is for 64 input channels");
  static constexpr int NW = (CIN == 32) ? 64 : 32;   // output columns per wave (18432 weights per wave)
  // WIDE: the four waves stand side by side (128 columns) and each takes both 32-pixel halves of the band, so that a
  // layer with more than 64 output channels loads its input once instead of once per 64 columns
  static constexpr int WGM = WIDE ? 1 : (CIN == 32) ? 4 : 2, WGN = 4 / WGM, TM = WIDE ? 2 : 1;
  static constexpr int BM = WGM * TM * 32, BN = WGN * NW;  // 128 x 64, 64 x 64 or 64 x 128
  static constexpr int PIX = CIN * 2;                 // bytes per pixel
  static constexpr int MAXSEG = 6;                    // 1 KiB load instructions per image row
  static constexpr int MAXBUF = 6;
  static constexpr int SP = NW + 8;                   // staging pitch (elements)
  static constexpr int STAGE_BYTES = 4 * 32 * SP * 2;
  static constexpr int THREADS = 512;                 // four compute waves + four loader waves
  static int image_bytes(int W, int TR) { return (2 * TR + 1) * (W + 2) * PIX; }
  static int lds_bytes(int W, int TR, int nbuf) { return nbuf * image_bytes(W, TR) + STAGE_BYTES + BN * 4; }
};

// LDS image rows hold pixel slots of CIN*2 bytes (slot 0 and slot W+1 are zero pads).  A byte at
// logical in-row offset `off` is stored at off ^ tile_swz_bits<CIN>(off): the 16-byte chunks of a
// pixel are permuted by bits of the slot index (which the permutation leaves unchanged, so it is
// its own inverse).  Reads that walk over every second slot then use all banks evenly, two lanes
// per bank group.
template <int CIN>
__device__ __forceinline__ uint32_t tile_swz_bits(uint32_t off) {
  if (CIN == 32) return ((off >> 8) & 3u) << 4;          // slot >> 2
  const uint32_t t = (off >> 8) & 7u;                    // slot >> 1
  return (((t & 1u) << 2) | (t >> 1)) << 4;              // rotated, so neighbours differ in the top bit
}

// The forward kernel's form for 64 channels.  A b128 operand read is served eight lanes at a time, and eight lanes
// run at full rate when their 16-byte chunks sit at eight different positions of the 128-byte pixel.  Consecutive
// lanes are consecutive output pixels, row after row of the band, so the key that permutes a pixel's chunks counts
// pixels the same way: slot pair + Wo * (image row / 2), i.e. lane number plus a constant for every tap.  (The
// in-row key alone repeats where a short output row wraps inside a group of eight lanes: 16 instead of 8 cycles
// per read at Wo = 10.)  `rowkey` = Wo * (row >> 1) of the LDS image row the byte belongs to.
template <int CIN>
__device__ __forceinline__ uint32_t fwd_swz_bits(uint32_t off, uint32_t rowkey) {
  if (CIN == 32) return tile_swz_bits<32>(off);
  return (((off >> 8) + rowkey) & 7u) << 4;
}

// AUX: cache policy of the band loads (LOAD_NT where a band shares few rows with its neighbours)
template <int CIN, int AUX, int WIDE = 0>
__global__ __launch_bounds__(512) void k_conv_fwd_tile(ConvTileArgs a) {
  typedef ConvTileShape<CIN, WIDE> S;
  constexpr int NW = S::NW, WGN = S::WGN, TN = NW / 32, TM = S::TM, PIX = S::PIX, SP = S::SP;
  constexpr int KC = CIN / 16;  // MFMA k-steps per tap
  constexpr int CPP = CIN / 8;  // 16-byte chunks per pixel
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int W = a.W, WP = W + 2, TR = a.TR, Wo = a.Wo, NBUF = a.nbuf;
  const int nrows = 2 * TR + 1, rowbytes = W * PIX, segs = (rowbytes + 1023) >> 10;
  const int image_bytes = nrows * WP * PIX;
  // tiles of this block: vb, vb + gridDim.x, ...
  const int vb = xcd_block((int)blockIdx.x, (int)gridDim.x);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / (int)gridDim.x + 1 : 0;

  // zero the pad pixels of all ring images once
  for (int i = tid; i < NBUF * nrows * 2 * CPP; i += S::THREADS) {
    const int chunk = i % CPP, side = (i / CPP) & 1, row = i / (2 * CPP);  // row over all images
    *reinterpret_cast<uint4*>(lds + (int64_t)row * WP * PIX + (side ? (W + 1) * PIX : 0) + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }

  if (wave >= 4) {
    // ------------------------------------------------------------------ loaders: span row r belongs to loader r % 4
    const int lw = wave - 4;
    const int ni = ((nrows - lw + 3) >> 2) * segs;  // this wave's loads per band
    // this lane's 16 bytes land at in-row offset PIX + sg*1024 + lane*16: it fetches what belongs there
    // (byte offset within the image row; depends on the row for 64 channels)
    auto src_off = [&](int sg, int row) {
      const uint32_t phys = PIX + sg * 1024 + lane * 16, logi = phys ^ fwd_swz_bits<CIN>(phys, (uint32_t)(Wo * (row >> 1)));
      return (sg < segs && (int)phys < (W + 1) * PIX) ? (int)logi - PIX : -1;  // -1 = none
    };
    int goff[S::MAXSEG];
#pragma unroll
    for (int sg = 0; sg < S::MAXSEG; ++sg) goff[sg] = src_off(sg, 0);
    int slot = 0;  // ring image the next issued band goes to
    auto issue = [&](int q) {
      const int t = vb + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int iy_lo = 2 * band * TR - 1;
      const char* src = reinterpret_cast<const char*>(a.in.ptr_uniform(img)) + (int64_t)iy_lo * rowbytes;
      char* dst = lds + slot * image_bytes + PIX;  // skip the left pad
      slot = slot + 1 == NBUF ? 0 : slot + 1;
      for (int row = lw; row < nrows; row += 4) {
        const int iy = iy_lo + row;
        const bool inside = iy >= 0 && iy < a.H;
#pragma unroll
        for (int sg = 0; sg < S::MAXSEG; ++sg)
          if (sg < segs) {
            const int go = (CIN == 32) ? goff[sg] : src_off(sg, row);
            const char* p = inside ? src + (int64_t)row * rowbytes + go : reinterpret_cast<const char*>(a.zpage) + lane * 16;
            if (go >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + row * WP * PIX + sg * 1024), 16, 0, AUX);
          }
      }
    };
    const int D = NBUF - 1;  // bands in flight
    for (int q = 0; q < D && q < nq; ++q) issue(q);
    for (int q = 0; q < nq; ++q) {
      vm_wait_dyn(min(D - 1, nq - 1 - q) * ni);  // band q has landed; the bands issued after it may still be in flight
      __builtin_amdgcn_s_barrier();
      if (q + D < nq) issue(q + D);      // into the slot the compute waves finished before this barrier
    }
    return;
  }

  // -------------------------------------------------------------------- compute waves
  const int wm = wave / WGN, wn = wave % WGN;
  char* const stage = lds + NBUF * image_bytes + wave * (32 * SP * 2);
  float* const bias_s = reinterpret_cast<float*>(lds + NBUF * image_bytes + S::STAGE_BYTES);
  const int nb0 = blockIdx.y * S::BN, n0 = nb0 + wn * NW;
  for (int i = tid; i < S::BN; i += 256) bias_s[i] = (nb0 + i < a.Cout) ? a.bias[nb0 + i] : 0.f;

  // this wave's weights, in MFMA operand layout: lane (column l32 of tile j, 8 k at h*8)
  bf16x8_t wr[9 * KC][TN];
#pragma unroll
  for (int s = 0; s < 9 * KC; ++s)
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + j * 32 + l32;
      wr[s][j] = (n < a.Cout) ? *reinterpret_cast<const bf16x8_t*>(a.w + (int64_t)n * (9 * CIN) + s * 16 + h * 8)
                              : __builtin_bit_cast(bf16x8_t, make_uint4(0u, 0u, 0u, 0u));
    }

  // this lane's output pixel(s) within a band, the LDS offset of the window corner (slot 2*ox of row
  // 2*oyl) and, per tap column v, the chunk permutation of slot 2*ox + v folded with the lane's k half
  // (for 64 channels the permutation also depends on the image row pair: rows 2*oyl, 2*oyl + 1 for the taps
  // u < 2, row 2*oyl + 2 for u = 2)
  constexpr int NU = (CIN == 32) ? 1 : 2;
  uint32_t abase[TM], hx[TM][NU][3];
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int r = (wm * TM + i) * 32 + l32;
    const bool in_band = r < TR * Wo;  // lanes beyond the band compute on pixel 0; never stored
    const int oyl = in_band ? r / Wo : 0, ox = in_band ? r - oyl * Wo : 0;
    abase[i] = (uint32_t)(((2 * oyl) * WP + 2 * ox) * PIX);
#pragma unroll
    for (int u2 = 0; u2 < NU; ++u2)
#pragma unroll
      for (int v = 0; v < 3; ++v)
        hx[i][u2][v] = (uint32_t)(h * 16) ^ fwd_swz_bits<CIN>((uint32_t)((2 * ox + v) * PIX), (uint32_t)(Wo * (oyl + u2)));
  }

  // the first tile's barrier also orders the pad fill and the bias table before their first use
  int slot = 0;
  for (int q = 0; q < nq; ++q) {
    const int t = vb + q * gridDim.x;
    __builtin_amdgcn_s_barrier();  // band q is in LDS
    const char* img_s = lds + slot * image_bytes;
    slot = slot + 1 == NBUF ? 0 : slot + 1;

    f32x16_t acc[TM][TN];  // starts at the bias of the lane's columns j*32 + g*8 + h*4 + 0..3
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 bv = *reinterpret_cast<const float4*>(bias_s + wn * NW + j * 32 + g * 8 + h * 4);
#pragma unroll
        for (int i = 0; i < TM; ++i) { acc[i][j][g * 4] = bv.x; acc[i][j][g * 4 + 1] = bv.y; acc[i][j][g * 4 + 2] = bv.z; acc[i][j][g * 4 + 3] = bv.w; }
      }
    // The operand reads run RD steps ahead of the MFMAs through a rotation of RD + 1 registers (step s = tap, 16-deep
    // chunk cc, pixel group i): with one compute wave per SIMD nothing else hides the LDS latency, and left to
    // itself the compiler keeps a single read in flight.  Logical chunk 2*cc + h of a slot sits at position
    // (2*cc + h) ^ f(slot, row) = (32*cc) ^ hx in bytes.
    constexpr int NS = 9 * KC * TM, RD = 3;
    auto operand = [&](int s) {
      const int i = s % TM, cc = (s / TM) % KC, tap = s / (TM * KC), u = tap / 3, v = tap - 3 * u;
      return *reinterpret_cast<const bf16x8_t*>(img_s + abase[i] + (u * WP + v) * PIX + ((uint32_t)(cc * 32) ^ hx[i][(NU == 2 && u == 2) ? 1 : 0][v]));
    };
    bf16x8_t av[RD + 1];
#pragma unroll
    for (int s = 0; s < RD; ++s) av[s] = operand(s);
#pragma unroll
    for (int s = 0; s < NS; ++s) {
      if (s + RD < NS) av[(s + RD) % (RD + 1)] = operand(s + RD);
      const int i = s % TM;
#pragma unroll
      for (int j = 0; j < TN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[s / TM][j], av[s % (RD + 1)], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);  // keep the read of step s + RD in front of the MFMA of step s
    }
    // ---- epilogue: bf16, ReLU; lane holds pixel l32 of the wave's pixel group i, columns j*32 + g*8 + h*4 + 0..3
    const int img = t / a.NB, band = t - img * a.NB;
    const int b = img / a.V, vw = img - b * a.V;
    const int rows_here = min(TR, a.Ho - band * TR);
    const int plim = rows_here * Wo;  // pixels of the band that exist
    bf16_t* dst = a.out + (int64_t)b * a.out_stride_b + (int64_t)vw * a.out_stride_v + (int64_t)band * TR * Wo * a.Cout;
    const uint32_t negw = nonzero_weights(h);
#pragma unroll
    for (int i = 0; i < TM; ++i) {
      const int p0 = (wm * TM + i) * 32;  // the group's first pixel (the strip is reused per group: a wave's LDS
                                          // accesses are served in order)
      uint32_t pw[TN];  // this lane's 16 sign bits of the pixel's 32-column group j
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        pw[j] = 0u;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const int cl = j * 32 + g * 8 + h * 4;
          uint2 o;
          o.x = relu_pack2bf(acc[i][j][g * 4], acc[i][j][g * 4 + 1]);
          o.y = relu_pack2bf(acc[i][j][g * 4 + 2], acc[i][j][g * 4 + 3]);
          *reinterpret_cast<uint2*>(stage + (l32 * SP + cl) * 2) = o;
          pw[j] |= nonzero4(o.x, o.y, negw) << (g * 8);
        }
      }
      if (a.bits) {
        // the other half of the columns sits in lane ^ 32; lanes 0..31 write the pixel's words
        const int wpp = (a.Cout + 31) >> 5, p = p0 + l32;
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const uint32_t word = or_with_lane_xor32(pw[j]);
          const int wi = (n0 >> 5) + j;
          if (h == 0 && p < plim && wi < wpp)
            a.bits[((int64_t)img * a.Ho * Wo + (int64_t)band * TR * Wo + p) * wpp + wi] = word;
        }
      }
      constexpr int CPRO = NW / 8;  // 16-byte chunks per staged row
#pragma unroll
      for (int e = 0; e < 32 * CPRO / 64; ++e) {
        const int ch = lane + 64 * e, rl = ch / CPRO, cg = ch - rl * CPRO;
        const int p = p0 + rl, n = n0 + cg * 8;
        if (p < plim && n < a.Cout)
          store_stream16(dst + (int64_t)p * a.Cout + n, *reinterpret_cast<const uint4*>(stage + (rl * SP + cg * 8) * 2));
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// Weight gradient of the same convolution: G[n][k] = sum over pixels p of dY[p][n] * X[win(p)][k],
// k = (u*3+v)*CIN + ci, with the same organisation.  A tile is (image, band of TR output rows); the
// loader waves copy the band's input rows (LDS image as above) and the band's dY pixels (64 output
// channels of this block, 128 bytes per pixel, NSTEP*16 pixels with zeros beyond the band) into a
// ring of nbuf buffers (three, or more where they fit: small bands need more of them in flight).  The contraction runs over pixels, 16 per MFMA step; both operands are
// read through ds_read_b64_tr_b16 (lane r of a 16-lane group supplies 4 consecutive channels of
// pixel r/4, lane i receives channel i of 4 pixels), the im2col being the per-lane pixel address.
// Compute wave w owns the 32-wide k-tiles w, w+4, ... of both 32-row n-tiles; the accumulators live
// in registers across all tiles of the block and leave once, as this block's fp32 partial
// [9*CIN][Cout] (partials are summed in a fixed order by the caller).  Wave 3 also accumulates the
// column sums of dY (the bias gradient) with an all-ones operand.
// dY pixels are 128 bytes apart; bit 6 of the offset is flipped for every second pixel pair so that
// the four pixels of one transposing read fall into different banks.
struct ConvWgradArgs {
  ImgAddr in;                 // layer input X, images [H][W][CIN], dense
  ImgAddr dy;                 // gradient of the layer output, images [Ho][Wo][Cout]
  const bf16_t* zpage;        // 1 KiB of zeros
  float* partial;             // [gridDim.x][9*CIN][Cout]
  float* bias_partial;        // [gridDim.x][Cout]
  int H, W, Ho, Wo, Cout;
  int TR, NB, ntiles, nstep;  // output rows per band, bands per image, nimg * NB, ceil(TR*Wo / 16)
  int nbuf;                   // ring buffers (3 .. MAXBUF)
};

template <int CIN>
struct ConvWgradShape {
  static constexpr int PIX = CIN * 2, KT = 9 * CIN / 32, KTW = (KT + 3) / 4;
  static constexpr int MAXSEG = 6, MAXSTEP = (CIN == 32) ? 8 : 4, MAXBUF = 6, THREADS = 512;
  static_assert(3 + 4 * (KTW - 1) >= KT, "wave 3's last accumulator pair must be free for the bias sums");
  static int image_bytes(int W, int TR) { return (2 * TR + 1) * (W + 2) * PIX; }
  static int buf_bytes(int W, int TR, int nstep) { return image_bytes(W, TR) + nstep * 16 * 128; }
  static int lds_bytes(int W, int TR, int nstep, int nbuf) { return nbuf * buf_bytes(W, TR, nstep) + 4 * 64 * 4; }
};

__device__ __forceinline__ bf16x8_t lds_read_tr8_2(const char* p_lo, const char* p_hi) {
  typedef short s16x4_t_ __attribute__((ext_vector_type(4)));
  struct { s16x4_t_ lo, hi; } v;
  v.lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t_ __attribute__((address_space(3)))*)(p_lo));
  v.hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4_t_ __attribute__((address_space(3)))*)(p_hi));
  return __builtin_bit_cast(bf16x8_t, v);
}

// NS > 0: the number of pixel steps per band is NS (known when the kernel is compiled), which lets the tile loop run
// without a branch and its operand reads ahead of the MFMAs; NS = 0: any number of steps up to MAXSTEP.
template <int CIN, int NS = 0>
__global__ __launch_bounds__(512) void k_conv_wgrad_tile(ConvWgradArgs a) {
  typedef ConvWgradShape<CIN> S;
  constexpr int PIX = S::PIX, KT = S::KT, KTW = S::KTW, MAXSTEP = S::MAXSTEP;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int W = a.W, WP = W + 2, TR = a.TR, Wo = a.Wo, nstep = NS ? NS : a.nstep, NBUF = a.nbuf;
  const int nrows = 2 * TR + 1, rowbytes = W * PIX, segs = (rowbytes + 1023) >> 10;
  const int image_bytes = nrows * WP * PIX, dy_bytes = nstep * 16 * 128, buf_bytes = image_bytes + dy_bytes;
  const int vb = xcd_block((int)blockIdx.x, (int)gridDim.x);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / (int)gridDim.x + 1 : 0;
  const int nb0 = blockIdx.y * 64;

  // zero the pad pixels of all ring images once
  for (int i = tid; i < NBUF * nrows * 2 * (PIX / 16); i += S::THREADS) {
    const int chunk = i % (PIX / 16), side = (i / (PIX / 16)) & 1, row = i / (2 * (PIX / 16));
    const int b = row / nrows, rr = row - b * nrows;
    *reinterpret_cast<uint4*>(lds + b * buf_bytes + (int64_t)rr * WP * PIX + (side ? (W + 1) * PIX : 0) + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }

  if (wave >= 4) {
    // ------------------------------------------------------------------ loaders
    // loader lw copies the image rows lw, lw+4, ... and the 1 KiB dY pieces lw, lw+4, ... of a band
    const int lw = wave - 4;
    const int ni = ((nrows - lw + 3) >> 2) * segs + ((nstep * 2 - lw + 3) >> 2);  // this wave's loads per band
    int xgoff[S::MAXSEG];
#pragma unroll
    for (int sg = 0; sg < S::MAXSEG; ++sg) {
      const uint32_t phys = PIX + sg * 1024 + lane * 16, logi = phys ^ tile_swz_bits<CIN>(phys);
      xgoff[sg] = (sg < segs && (int)phys < (W + 1) * PIX) ? (int)logi - PIX : -1;
    }
    int slot = 0;  // ring buffer the next issued band goes to
    auto issue = [&](int q) {
      const int t = vb + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int iy_lo = 2 * band * TR - 1;
      const char* xsrc = reinterpret_cast<const char*>(a.in.ptr_uniform(img)) + (int64_t)iy_lo * rowbytes;
      const int plim = min(TR, a.Ho - band * TR) * Wo;  // pixels of the band that exist
      const bf16_t* dsrc = a.dy.ptr_uniform(img) + (int64_t)band * TR * Wo * a.Cout + nb0;
      char* buf = lds + slot * buf_bytes;
      slot = slot + 1 == NBUF ? 0 : slot + 1;
      const char* zp = reinterpret_cast<const char*>(a.zpage) + lane * 16;
      for (int row = lw; row < nrows; row += 4) {
        const int iy = iy_lo + row;
        const bool inside = iy >= 0 && iy < a.H;
#pragma unroll
        for (int sg = 0; sg < S::MAXSEG; ++sg)
          if (sg < segs) {
            const char* p = inside ? xsrc + (int64_t)row * rowbytes + xgoff[sg] : zp;
            if (xgoff[sg] >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(buf + row * WP * PIX + PIX + sg * 1024), 16, 0, LOAD_NT);
          }
      }
      for (int j = lw; j < nstep * 2; j += 4) {  // 1 KiB = 8 pixels of 128 bytes
        const uint32_t phys = j * 1024 + lane * 16, logi = phys ^ (((phys >> 8) & 1u) << 6);
        const int p_ = (int)(logi >> 7), cb = (int)(logi & 127u);
        const bool ok = p_ < plim && nb0 + (cb >> 1) < a.Cout;
        const char* p = ok ? reinterpret_cast<const char*>(dsrc + (int64_t)p_ * a.Cout) + cb : zp;
        __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(buf + image_bytes + j * 1024), 16, 0, LOAD_NT);
      }
    };
    const int D = NBUF - 1;  // bands in flight
    for (int q = 0; q < D && q < nq; ++q) issue(q);
    for (int q = 0; q < nq; ++q) {
      vm_wait_dyn(min(D - 1, nq - 1 - q) * ni);  // band q has landed; the bands issued after it may still be in flight
      __builtin_amdgcn_s_barrier();
      if (q + D < nq) issue(q + D);
    }
    __builtin_amdgcn_s_barrier();  // pairs with the compute waves' barrier before the bias reduction
    return;
  }

  // -------------------------------------------------------------------- compute waves
  const int g = lane >> 4, r16 = lane & 15;
  const int scolb = (16 * (g & 1) + 4 * (r16 & 3)) * 2;  // byte offset of this lane's 4 source channels in a 32-channel tile
  // per step and half (pixels +0..3 / +4..7 of the lane's group): source addresses within a ring buffer
  uint32_t xb[MAXSTEP][2][2];  // image: pixel (2*oyl, 2*ox) with the chunk permutation of tap columns v < 2 / v = 2
  uint32_t db[MAXSTEP][2];     // dY: pixel p, n-tile 0
#pragma unroll
  for (int s = 0; s < MAXSTEP; ++s)
#pragma unroll
    for (int hf = 0; hf < 2; ++hf) {
      int p = s * 16 + 8 * (g >> 1) + (r16 >> 2) + 4 * hf;
      const uint32_t dl = (uint32_t)(p * 128 + scolb);
      db[s][hf] = (uint32_t)image_bytes + (dl ^ (((dl >> 8) & 1u) << 6));
      if (p >= TR * Wo) p = 0;  // its dY is zero; any finite pixel will do
      const int oyl = p / Wo, ox = p - oyl * Wo;
      const uint32_t inrow = (uint32_t)(2 * ox * PIX + scolb), rowb = (uint32_t)(2 * oyl * WP * PIX);
      xb[s][hf][0] = rowb + (inrow ^ tile_swz_bits<CIN>(inrow));
      xb[s][hf][1] = rowb + (inrow ^ tile_swz_bits<CIN>(inrow + 2 * PIX));
    }

  f32x16_t acc[KTW][2];  // wave 3 has no k-tile for t = KTW-1: that pair holds the bias sums
#pragma unroll
  for (int t = 0; t < KTW; ++t)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][i][e] = 0.f;
  const bf16x8_t ones = __builtin_bit_cast(bf16x8_t, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));
  // byte offset of k-tile kt within the window: tap (u, v) and, for 64 channels, the pixel half
  uint32_t tapc[KTW]; bool tapv2[KTW], taphi[KTW];
#pragma unroll
  for (int t = 0; t < KTW; ++t) {
    // (a wave without a k-tile for t = KTW-1 reads its first one again where the loop has no branch: the product
    // lands in an accumulator that is never stored, or is replaced by the bias operand)
    const int kt = (wave + 4 * t < KT) ? wave + 4 * t : wave, tap = kt / (CIN / 32), u = tap / 3, v = tap - 3 * u;
    tapc[t] = (uint32_t)((u * WP + v) * PIX); tapv2[t] = v == 2; taphi[t] = (CIN == 64) && (kt & 1);
  }

  int slot = 0;
  for (int q = 0; q < nq; ++q) {
    __builtin_amdgcn_s_barrier();  // band q is in LDS (the first one also orders the pad fill)
    const char* buf = lds + slot * buf_bytes;
    slot = slot + 1 == NBUF ? 0 : slot + 1;
    if constexpr (NS > 0) {
      // The operand reads run ahead of the MFMAs (the window operand RD k-tiles, the dY operand a whole pixel
      // step): with one compute wave per SIMD nothing else hides the LDS latency, and left to itself the compiler
      // waits for each read right where it is used.  No branch inside: every wave runs KTW k-tiles per step.
      constexpr int NU = NS * KTW, RD = 2;
      bf16x8_t aq[2][2], bq[RD + 1];
      const uint32_t bias_sel = (wave == 3) ? 0xffffffffu : 0u;  // wave 3's last k-tile is the bias column
      auto read_a = [&](int s_) __attribute__((always_inline)) {
        aq[s_ & 1][0] = lds_read_tr8_2(buf + db[s_][0], buf + db[s_][1]);
        aq[s_ & 1][1] = lds_read_tr8_2(buf + (db[s_][0] ^ 64u), buf + (db[s_][1] ^ 64u));
      };
      auto read_b = [&](int u) __attribute__((always_inline)) {
        const int s_ = u / KTW, t_ = u % KTW;
        uint32_t o0 = tapv2[t_] ? xb[s_][0][1] : xb[s_][0][0], o1 = tapv2[t_] ? xb[s_][1][1] : xb[s_][1][0];
        const uint32_t hi = taphi[t_] ? 64u : 0u;
        o0 ^= hi; o1 ^= hi;
        bq[u % (RD + 1)] = lds_read_tr8_2(buf + o0 + tapc[t_], buf + o1 + tapc[t_]);
      };
      read_a(0);
#pragma unroll
      for (int u = 0; u < RD && u < NU; ++u) read_b(u);
#pragma unroll
      for (int u = 0; u < NU; ++u) {
        const int s_ = u / KTW, t = u % KTW;
        if (t == 0 && s_ + 1 < NS) read_a(s_ + 1);
        if (u + RD < NU) read_b(u + RD);
        bf16x8_t bop = bq[u % (RD + 1)];
        if (t == KTW - 1) {
          const uint4 bu = __builtin_bit_cast(uint4, bop), on = __builtin_bit_cast(uint4, ones);
          bop = __builtin_bit_cast(bf16x8_t, make_uint4((bu.x & ~bias_sel) | (on.x & bias_sel), (bu.y & ~bias_sel) | (on.y & bias_sel),
                                                         (bu.z & ~bias_sel) | (on.z & bias_sel), (bu.w & ~bias_sel) | (on.w & bias_sel)));
        }
        acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[s_ & 1][0], bop, acc[t][0], 0, 0, 0);
        acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aq[s_ & 1][1], bop, acc[t][1], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // keep the reads in front of the MFMAs they run ahead of
      }
    } else {
#pragma unroll
    for (int s = 0; s < MAXSTEP; ++s) {
      if (s < nstep) {
        const bf16x8_t a0 = lds_read_tr8_2(buf + db[s][0], buf + db[s][1]);
        const bf16x8_t a1 = lds_read_tr8_2(buf + (db[s][0] ^ 64u), buf + (db[s][1] ^ 64u));
#pragma unroll
        for (int t = 0; t < KTW; ++t) {
          if (wave + 4 * t < KT) {
            uint32_t o0 = tapv2[t] ? xb[s][0][1] : xb[s][0][0], o1 = tapv2[t] ? xb[s][1][1] : xb[s][1][0];
            if (taphi[t]) { o0 ^= 64u; o1 ^= 64u; }
            const bf16x8_t b = lds_read_tr8_2(buf + o0 + tapc[t], buf + o1 + tapc[t]);
            acc[t][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b, acc[t][0], 0, 0, 0);
            acc[t][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b, acc[t][1], 0, 0, 0);
          }
        }
        if (wave == 3 && a.bias_partial) {
          acc[KTW - 1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, ones, acc[KTW - 1][0], 0, 0, 0);
          acc[KTW - 1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, ones, acc[KTW - 1][1], 0, 0, 0);
        }
      }
    }
    }
  }
  // ---- this block's partial sums: acc[t][i][e] = G[n][k], k = (wave+4t)*32 + lane%32, n = nb0 + i*32 + (e/4)*8 + (lane/32)*4 + e%4.
  // The partial is stored k-major ([9*CIN][Cout]) so that a lane's four consecutive n leave as one 16-byte store
  // (a quarter of the store instructions; the reduction kernel transposes back).
  const int K = 9 * CIN;
  float* P = a.partial + (int64_t)blockIdx.x * a.Cout * K;
#pragma unroll
  for (int t = 0; t < KTW; ++t) {
    const int kt = wave + 4 * t, k = kt * 32 + (lane & 31);
    if (kt < KT) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
          const int n = nb0 + i * 32 + g4 * 8 + (lane >> 5) * 4;
          if (n < a.Cout)  // Cout is a multiple of 8
            *reinterpret_cast<float4*>(P + (int64_t)k * a.Cout + n) = make_float4(acc[t][i][g4 * 4], acc[t][i][g4 * 4 + 1], acc[t][i][g4 * 4 + 2], acc[t][i][g4 * 4 + 3]);
        }
    }
  }
  __builtin_amdgcn_s_barrier();
  if (wave == 3 && a.bias_partial && (lane & 31) == 0) {
    // every column of the pair holds the same sums; lanes 0 and 32 cover the 64 rows between them
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int n = nb0 + i * 32 + (e >> 2) * 8 + (lane >> 5) * 4 + (e & 3);
        if (n < a.Cout) a.bias_partial[(int64_t)blockIdx.x * a.Cout + n] = acc[KTW - 1][i][e];
      }
  }
}
