// 3x3 stride-2 pad-1 convolution forward for 32 or 64 input channels, organised around what is
// scarce on the CU for this shape: bytes in flight per CU and vector-ALU issue slots, not MFMA
// cycles.
//
//  * Persistent blocks walk over tiles = (image, band of TR output rows).  The band's input rows
//    (2*TR+1 of them, one contiguous span of the channel-last image) are copied as they are into
//    an LDS image; the im2col gather happens at LDS-read time, where a tap is a constant byte
//    offset from the lane's window corner.  Every input byte crosses the memory path once per block.
//  * The copy is done by four extra waves with loads that write LDS directly (global_load_lds_dwordx4,
//    lane l's 16 bytes land at the instruction's LDS base + 16*l), into a ring of three images:
//    two bands are in flight while one is computed.  (One wave alone sustains only about one such
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
  int V, H, W, Ho, Wo, Cout;
  int TR, NB, ntiles;         // output rows per band, bands per image, nimg * NB
};

template <int CIN>
struct ConvTileShape {
  static constexpr int NW = (CIN == 32) ? 64 : 32;   // output columns per wave (18432 weights per wave)
  static constexpr int WGM = (CIN == 32) ? 4 : 2, WGN = 4 / WGM;
  static constexpr int BM = WGM * 32, BN = WGN * NW;  // 128 x 64 or 64 x 64
  static constexpr int PIX = CIN * 2;                 // bytes per pixel
  static constexpr int MAXSEG = 6;                    // 1 KiB load instructions per image row
  static constexpr int NBUF = 3;
  static constexpr int SP = NW + 8;                   // staging pitch (elements)
  static constexpr int STAGE_BYTES = 4 * 32 * SP * 2;
  static constexpr int THREADS = 512;                 // four compute waves + four loader waves
  static int image_bytes(int W, int TR) { return (2 * TR + 1) * (W + 2) * PIX; }
  static int lds_bytes(int W, int TR) { return NBUF * image_bytes(W, TR) + STAGE_BYTES + BN * 4; }
};

// wait until at most n (wave-uniform, < 64) of this wave's vector-memory operations are outstanding
__device__ __forceinline__ void vm_wait_dyn(int n) {
  switch (n) {
#define VMW(i) case i: vm_wait<i>(); break;
#define VMW8(b) VMW(b) VMW(b + 1) VMW(b + 2) VMW(b + 3) VMW(b + 4) VMW(b + 5) VMW(b + 6) VMW(b + 7)
    VMW8(0) VMW8(8) VMW8(16) VMW8(24) VMW8(32) VMW8(40) VMW8(48) VMW8(56)
#undef VMW8
#undef VMW
    default: vm_wait<0>(); break;
  }
}

template <int CIN>
__global__ __launch_bounds__(512) void k_conv_fwd_tile(ConvTileArgs a) {
  typedef ConvTileShape<CIN> S;
  constexpr int NW = S::NW, WGN = S::WGN, TN = NW / 32, PIX = S::PIX, SP = S::SP, NBUF = S::NBUF;
  constexpr int KC = CIN / 16;  // MFMA k-steps per tap
  constexpr int CPP = CIN / 8;  // 16-byte chunks per pixel
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int W = a.W, WP = W + 2, TR = a.TR, Wo = a.Wo;
  const int nrows = 2 * TR + 1, rowbytes = W * PIX, segs = (rowbytes + 1023) >> 10;
  const int image_bytes = nrows * WP * PIX;
  // tiles of this block: blockIdx.x, + gridDim.x, ...
  const int nq = (a.ntiles > (int)blockIdx.x) ? (a.ntiles - 1 - (int)blockIdx.x) / (int)gridDim.x + 1 : 0;
  // chunk permutation of the pixel in slot xs (slot 0 is the left pad)
  auto swz = [](int xs) -> int { return (CIN == 32) ? ((xs >> 2) & 3) : ((xs >> 1) & 7); };

  // zero the pad pixels of all ring images once
  for (int i = tid; i < NBUF * nrows * 2 * CPP; i += S::THREADS) {
    const int chunk = i % CPP, side = (i / CPP) & 1, row = i / (2 * CPP);  // row over all images
    *reinterpret_cast<uint4*>(lds + (int64_t)row * WP * PIX + (side ? (W + 1) * PIX : 0) + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }

  if (wave >= 4) {
    // ------------------------------------------------------------------ loaders: span row r belongs to loader r % 4
    const int lw = wave - 4;
    const int ni = ((nrows - lw + 3) >> 2) * segs;  // this wave's loads per band
    int goff[S::MAXSEG];  // byte offset within an image row of the chunk this lane fetches, -1 = none
#pragma unroll
    for (int sg = 0; sg < S::MAXSEG; ++sg) {
      const int L = sg * 64 + lane, xi = L / CPP, cip = L - xi * CPP;
      goff[sg] = (sg < segs && L < W * CPP) ? (xi * CPP + (cip ^ swz(xi + 1))) * 16 : -1;
    }
    auto issue = [&](int q) {
      const int t = blockIdx.x + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int iy_lo = 2 * band * TR - 1;
      const char* src = reinterpret_cast<const char*>(a.in.ptr(img)) + (int64_t)iy_lo * rowbytes;
      char* dst = lds + (q % NBUF) * image_bytes + PIX;  // skip the left pad
      for (int row = lw; row < nrows; row += 4) {
        const int iy = iy_lo + row;
        const bool inside = iy >= 0 && iy < a.H;
#pragma unroll
        for (int sg = 0; sg < S::MAXSEG; ++sg)
          if (sg < segs) {
            const char* p = inside ? src + (int64_t)row * rowbytes + goff[sg] : reinterpret_cast<const char*>(a.zpage) + lane * 16;
            if (goff[sg] >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + row * WP * PIX + sg * 1024), 16, 0, 0);
          }
      }
    };
    if (nq > 0) issue(0);
    if (nq > 1) issue(1);
    __builtin_amdgcn_s_barrier();  // pad fill done (matches the compute waves' first barrier)
    for (int q = 0; q < nq; ++q) {
      vm_wait_dyn(q + 1 < nq ? ni : 0);  // band q has landed; band q+1 may still be in flight
      __builtin_amdgcn_s_barrier();
      if (q + 2 < nq) issue(q + 2);      // into the slot the compute waves finished before this barrier
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

  // this lane's output pixel within a band, the LDS offset of its window corner (slot 2*ox of row
  // 2*oyl) and, per tap column v, the chunk permutation of slot 2*ox + v folded with the lane's k half
  const int r = wm * 32 + l32;
  const bool in_band = r < TR * Wo;  // lanes beyond the band compute on pixel 0; never stored
  const int oyl = in_band ? r / Wo : 0, ox = in_band ? r - oyl * Wo : 0;
  const uint32_t abase = (uint32_t)(((2 * oyl) * WP + 2 * ox) * PIX);
  uint32_t hx[3];
#pragma unroll
  for (int v = 0; v < 3; ++v) hx[v] = (uint32_t)((h ^ swz(2 * ox + v)) * 16);

  __builtin_amdgcn_s_barrier();  // pad fill and bias table done
  for (int q = 0; q < nq; ++q) {
    const int t = blockIdx.x + q * gridDim.x;
    __builtin_amdgcn_s_barrier();  // band q is in LDS
    const char* img_s = lds + (q % NBUF) * image_bytes;

    f32x16_t acc[TN];
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[j][e] = 0.f;
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
      for (int v = 0; v < 3; ++v) {
        const char* ap = img_s + abase + (u * WP + v) * PIX;
#pragma unroll
        for (int cc = 0; cc < KC; ++cc) {
          // logical chunk 2*cc + h sits at position (2*cc + h) ^ f(slot) = (32*cc) ^ hx[v] in bytes
          const bf16x8_t av = *reinterpret_cast<const bf16x8_t*>(ap + ((uint32_t)(cc * 32) ^ hx[v]));
#pragma unroll
          for (int j = 0; j < TN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[(u * 3 + v) * KC + cc][j], av, acc[j], 0, 0, 0);
        }
      }
    // ---- epilogue: bias, ReLU, bf16; lane holds pixel l32 of the wave, columns j*32 + g*8 + h*4 + 0..3
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = j * 32 + g * 8 + h * 4;
        const float4 bv = *reinterpret_cast<const float4*>(bias_s + wn * NW + cl);
        uint2 o;
        o.x = pack2bf(fmaxf(acc[j][g * 4] + bv.x, 0.f), fmaxf(acc[j][g * 4 + 1] + bv.y, 0.f));
        o.y = pack2bf(fmaxf(acc[j][g * 4 + 2] + bv.z, 0.f), fmaxf(acc[j][g * 4 + 3] + bv.w, 0.f));
        *reinterpret_cast<uint2*>(stage + (l32 * SP + cl) * 2) = o;
      }
    {
      const int img = t / a.NB, band = t - img * a.NB;
      const int b = img / a.V, vw = img - b * a.V;
      const int rows_here = min(TR, a.Ho - band * TR);
      const int plim = rows_here * Wo;  // pixels of the band that exist
      bf16_t* dst = a.out + (int64_t)b * a.out_stride_b + (int64_t)vw * a.out_stride_v + (int64_t)band * TR * Wo * a.Cout;
      constexpr int CPRO = NW / 8;  // 16-byte chunks per staged row
#pragma unroll
      for (int i = 0; i < 32 * CPRO / 64; ++i) {
        const int ch = lane + 64 * i, rl = ch / CPRO, cg = ch - rl * CPRO;
        const int p = wm * 32 + rl, n = n0 + cg * 8;
        if (p < plim && n < a.Cout)
          *reinterpret_cast<uint4*>(dst + (int64_t)p * a.Cout + n) = *reinterpret_cast<const uint4*>(stage + (rl * SP + cg * 8) * 2);
      }
    }
  }
}
