// Transposed convolution (input gradient of a 3x3 stride-2 pad-1 convolution) from 128 gradient
// channels to 64 result channels, organised like conv_dgrad_tile.hip.h: quads (2x2 blocks of
// result pixels) are the rows of the product, a quad's four dY pixels are read once from an LDS
// image of the band and meet the taps of the four pixel classes in registers, the result is staged
// in LDS and leaves, masked, as 16-byte segments of the band's contiguous span.
//
// What is different: 9 taps x 128 x 64 weights are twice the registers two compute waves have, so
// there are four, and the contraction over the gradient channels is split between them: wave
// (wn, kh) holds the taps' weights for result channels 32 wn .. + 31 and gradient channels
// 64 kh .. + 63 (144 registers) and stages its partial sum, rounded to bf16, in a staging area of
// its half; three finishing waves add the halves (in fp32), apply the ReLU mask of the stored
// activation (sign-bit words) and write (some sixty vector-ALU instructions per 16 bytes: the role
// that needs the waves).  One loader wave copies the band's dY rows (256 bytes per
// pixel, 1 KiB per load) into a ring of three LDS images; the 16-byte chunks of each 128-byte half
// of a pixel are permuted by slot + Wo * row, which numbers a wave's lanes consecutively across the
// short rows of such a layer, so that any eight consecutive lanes read eight different chunk
// positions.  Two barriers per tile order the three roles; the finishing waves work one tile
// behind the compute waves (double-buffered staging) and fetch their mask words two tiles ahead.
#pragma once
#include "conv_dgrad_tile.hip.h"

struct ConvDgradK2Shape {
  static constexpr int CI = 64, CO = 128, PB = CO * 2, BQ = 64, MT = 2, NBUF = 3, THREADS = 512, MAXSEG = 6;
  static constexpr int NFT = 192, MAXCH = 8;  // finishing threads, 16-byte chunks per finishing thread and tile
  static int dyimg_bytes(int Wo, int TQ) { return (TQ + 1) * (Wo + 1) * PB; }
  static int stage_bytes(int W, int TQ) { return 2 * TQ * W * CI * 2; }
  static int lds_bytes(int W, int Wo, int TQ) { return NBUF * dyimg_bytes(Wo, TQ) + 4 * stage_bytes(W, TQ); }
};

// permutation of the 16-byte chunks within each 128-byte half of a 256-byte dY pixel: `slot` in its row, `row` of the LDS image
__device__ __forceinline__ uint32_t dy2_swz_bits(int slot, int row, int Wo) { return (uint32_t)((slot + Wo * row) & 7) << 4; }

// the sum of two vectors of eight bf16, formed in fp32 and rounded once
__device__ __forceinline__ uint4 add_bf16x8(const uint4& x, const uint4& y) {
  auto add2 = [](uint32_t p, uint32_t q) -> uint32_t {
    const float lo = __uint_as_float(p << 16) + __uint_as_float(q << 16);
    const float hi = __uint_as_float(p & 0xffff0000u) + __uint_as_float(q & 0xffff0000u);
    return pack2bf(lo, hi);
  };
  return make_uint4(add2(x.x, y.x), add2(x.y, y.y), add2(x.z, y.z), add2(x.w, y.w));
}

__global__ __launch_bounds__(512) void k_conv_dgrad_k2_tile(ConvDgradArgs a) {
  typedef ConvDgradK2Shape S;
  constexpr int CI = S::CI, CO = S::CO, PB = S::PB, CC = 4, NBUF = S::NBUF, MT = S::MT;  // CC: 16-deep steps over a wave's 64 gradient channels
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int W = a.W, Wo = a.Wo, TQ = a.TQ;
  const int RP = (Wo + 1) * PB;  // dY image row pitch
  const int dyimg_bytes = (TQ + 1) * RP;
  const int stage_bytes = 2 * TQ * W * CI * 2;
  char* const stage0 = lds + NBUF * dyimg_bytes;  // [tile parity][gradient-channel half][stage_bytes]
  const int vb = xcd_block((int)blockIdx.x, (int)gridDim.x);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / (int)gridDim.x + 1 : 0;

  // zero the right pad slot of every dY image row once
  for (int i = tid; i < NBUF * (TQ + 1) * (PB / 16); i += S::THREADS) {
    const int chunk = i & (PB / 16 - 1), row = i / (PB / 16);
    *reinterpret_cast<uint4*>(lds + row * RP + Wo * PB + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }

  if (wave == 4) {
    // ------------------------------------------------------------------ loader (a quarter of a tile's time is enough for its loads)
    const int rowbytes = Wo * PB, segs = (rowbytes + 1023) >> 10;
    const int ni = (TQ + 1) * segs;  // loads per band
    auto issue = [&](int q) __attribute__((always_inline)) {
      const int t = vb + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int oy_lo = band * TQ;
      const char* src = reinterpret_cast<const char*>(a.dy.ptr_uniform(img)) + (int64_t)oy_lo * rowbytes;
      char* dst = lds + (q % NBUF) * dyimg_bytes;
      for (int row = 0; row <= TQ; ++row) {
        const bool inside = oy_lo + row < a.Ho;
#pragma unroll
        for (int sg = 0; sg < S::MAXSEG; ++sg)
          if (sg < segs) {
            // this lane's 16 bytes land at in-row offset sg*1024 + lane*16: it fetches what belongs there
            const uint32_t phys = sg * 1024 + lane * 16, logi = phys ^ dy2_swz_bits((int)(phys >> 8), row, Wo);
            const char* p = inside ? src + (int64_t)row * rowbytes + logi : reinterpret_cast<const char*>(a.zpage) + lane * 16;
            if ((int)phys < rowbytes) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + row * RP + sg * 1024), 16, 0, LOAD_NT);
          }
      }
    };
    if (nq > 0) issue(0);
    if (nq > 1) issue(1);
    for (int q = 0; q < nq; ++q) {
      vm_wait_dyn(q + 1 < nq ? ni : 0);  // band q has landed
      __builtin_amdgcn_s_barrier();      // A(q)
      if (q + 2 < nq) issue(q + 2);
      __builtin_amdgcn_s_barrier();      // B(q)
    }
    return;
  }

  if (wave >= 5) {
    // ------------------------------------------------------------------ finishing waves: thread et of 192 takes the chunks et, et + 192, ...
    const int et = tid - 320;
    const int nchunk = stage_bytes >> 4;
    // two register sets: the mask of tile q+1 is fetched while tile q-1 is finished
    uint32_t mk[2][S::MAXCH];      // the word holding a chunk's eight mask bits
    int64_t band_off[2] = {0, 0};  // element offset of the set's band within dx
    int nvalid[2] = {0, 0};        // its chunks that lie inside the image
    auto load_mask = [&](int q, auto setc) __attribute__((always_inline)) {
      constexpr int SET = decltype(setc)::value;
      const int t = vb + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int b = img / a.V, vw = img - b * a.V;
      const int rows = min(2 * TQ, a.H - 2 * band * TQ);
      band_off[SET] = (int64_t)b * a.x_stride_b + (int64_t)vw * a.x_stride_v + (int64_t)(2 * band * TQ) * W * CI;
      nvalid[SET] = rows * W * CI / 8;
      // mask words of the band: pixel (band-linear) c / (CI/8), word (c % (CI/8)) / 4
      const uint32_t* wb = a.xbits + ((int64_t)img * a.H + 2 * band * TQ) * W * (CI / 32);
#pragma unroll
      for (int i = 0; i < S::MAXCH; ++i) {
        const int c = et + S::NFT * i;
        uint32_t off = (uint32_t)(c >> 2) * 4u;  // four chunks (32 channels) per word
        asm volatile("" : "+v"(off));              // (keeps per-chunk 64-bit addresses from being carried across the tile loop)
        mk[SET][i] = (c < nchunk && c < nvalid[SET]) ? *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(wb) + off) : 0u;
      }
    };
    auto finish = [&](int q, auto setc) __attribute__((always_inline)) {  // tile q was loaded into set q & 1
      constexpr int SET = decltype(setc)::value;
      const char* st = stage0 + (q & 1) * 2 * stage_bytes;
      vm_wait<0>();  // one wait for everything outstanding (this set's mask words and the younger set's)
#pragma unroll
      for (int i = 0; i < S::MAXCH; ++i) {
        const int c = et + S::NFT * i;
        if (c < nchunk && c < nvalid[SET]) {
          const uint32_t L = (uint32_t)c * 16u, ph = L ^ tile_swz_bits<CI>(L);
          uint4 v = add_bf16x8(*reinterpret_cast<const uint4*>(st + ph), *reinterpret_cast<const uint4*>(st + stage_bytes + ph));
          const uint32_t b8 = mk[SET][i] >> ((c & 3) * 8);  // this chunk's eight bits
          v.x &= keep_pair(b8, 0); v.y &= keep_pair(b8, 1); v.z &= keep_pair(b8, 2); v.w &= keep_pair(b8, 3);
          uint32_t off = L;
          asm volatile("" : "+v"(off));
          store_stream16(reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(a.dx + band_off[SET]) + off), v);
        }
      }
    };
    typedef std::integral_constant<int, 0> set0;
    typedef std::integral_constant<int, 1> set1;
    auto step = [&](int q, auto par) __attribute__((always_inline)) {  // q & 1 == par
      constexpr int P = decltype(par)::value;
      typedef std::integral_constant<int, 1 - P> other;
      __builtin_amdgcn_s_barrier();  // A(q)
      if (q > 0) {
        finish(q - 1, other());
        if (q + 1 < nq) load_mask(q + 1, other());
      }
      __builtin_amdgcn_s_barrier();  // B(q): tile q is staged
    };
    if (nq > 0) load_mask(0, set0());
    if (nq > 1) load_mask(1, set1());
    for (int q = 0; q < nq; q += 2) {
      step(q, set0());
      if (q + 1 < nq) step(q + 1, set1());
    }
    if (nq > 0) { if ((nq - 1) & 1) finish(nq - 1, set1()); else finish(nq - 1, set0()); }
    return;
  }

  // -------------------------------------------------------------------- compute waves
  const int l32 = lane & 31, h = lane >> 5;
  const int wn = wave & 1, kh = wave >> 1;
  // weights: lane (column ci = wn*32 + l32, 8 co at kh*64 + cc*16 + h*8) of tap s
  bf16x8_t wr[9][CC];
#pragma unroll
  for (int s = 0; s < 9; ++s)
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
      wr[s][cc] = *reinterpret_cast<const bf16x8_t*>(a.wt + ((int64_t)s * CI + wn * 32 + l32) * CO + kh * 64 + cc * 16 + h * 8);

  for (int q = 0; q < nq; ++q) {
    const int t = vb + q * gridDim.x;
    const int band = t % a.NB;
    __builtin_amdgcn_s_barrier();  // A(q): band q is in LDS, staging buffer q&1 is free
    char* st = stage0 + ((q & 1) * 2 + kh) * stage_bytes;
    const int rows_here = a.H - 2 * band * TQ;  // image rows left from the band's first row
    const int mtn = (TQ * Wo + 31) >> 5;  // 32-quad groups of a band (at most MT)
#pragma unroll 1
    for (int mt = 0; mt < mtn; ++mt) {
      // this lane's quad of the group (lanes beyond the band work on quad 0 and store nothing)
      const int qi = mt * 32 + l32;
      const bool in_band = qi < TQ * Wo;
      const int al = in_band ? qi / Wo : 0, b = in_band ? qi - al * Wo : 0;
      const char* img_s = lds + (q % NBUF) * dyimg_bytes + al * RP + b * PB + kh * 128;
      uint32_t hx[2][2];  // [row offset][column offset] of the quad's four dY pixels
#pragma unroll
      for (int dyo = 0; dyo < 2; ++dyo)
#pragma unroll
        for (int dxo = 0; dxo < 2; ++dxo) hx[dyo][dxo] = (uint32_t)(h * 16) ^ dy2_swz_bits(b + dxo, al + dyo, Wo);
      f32x16_t acc[4];
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
      // the four dY pixels are fetched one pixel (all its channel chunks) ahead of the MFMAs that use them
      bf16x8_t av[2][CC];
      auto fetch = [&](int pi, bf16x8_t (&dst)[CC]) __attribute__((always_inline)) {
        const int dyo = pi >> 1, dxo = pi & 1;
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
          dst[cc] = *reinterpret_cast<const bf16x8_t*>(img_s + dyo * RP + dxo * PB + ((uint32_t)(cc * 32) ^ hx[dyo][dxo]));
      };
      fetch(0, av[0]);
#pragma unroll
      for (int pi = 0; pi < 4; ++pi) {
        if (pi + 1 < 4) fetch(pi + 1, av[(pi + 1) & 1]);
        const bf16x8_t (&x)[CC] = av[pi & 1];
        // class (py, px) takes tap u = py ? (dyo ? 0 : 2) : 1 from row offset dyo (even rows only from dyo = 0), same for columns
#pragma unroll
        for (int cc = 0; cc < CC; ++cc) {
          if (pi == 0) {
            acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[1 * 3 + 1][cc], x[cc], acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[1 * 3 + 2][cc], x[cc], acc[1], 0, 0, 0);
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[2 * 3 + 1][cc], x[cc], acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[2 * 3 + 2][cc], x[cc], acc[3], 0, 0, 0);
          } else if (pi == 1) {
            acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[1 * 3 + 0][cc], x[cc], acc[1], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[2 * 3 + 0][cc], x[cc], acc[3], 0, 0, 0);
          } else if (pi == 2) {
            acc[2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[0 * 3 + 1][cc], x[cc], acc[2], 0, 0, 0);
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[0 * 3 + 2][cc], x[cc], acc[3], 0, 0, 0);
          } else {
            acc[3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wr[0 * 3 + 0][cc], x[cc], acc[3], 0, 0, 0);
          }
        }
      }
      // ---- stage: lane holds, per class, columns wn*32 + g*8 + h*4 + 0..3 of its pixel
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool col_ok = in_band && ((c & 1) == 0 || 2 * b + 1 < W);
        if (col_ok && 2 * al + (c >> 1) < rows_here) {
          // staged position of pixel class c = py*2 + px, columns wn*32 + h*4 + g*8
          const uint32_t L = (uint32_t)((((2 * al + (c >> 1)) * W + 2 * b + (c & 1)) * CI + wn * 32 + h * 4) * 2);
          const uint32_t sp = L ^ tile_swz_bits<CI>(L);
#pragma unroll
          for (int g = 0; g < 4; ++g) {
            uint2 o;
            o.x = pack2bf(acc[c][g * 4], acc[c][g * 4 + 1]);
            o.y = pack2bf(acc[c][g * 4 + 2], acc[c][g * 4 + 3]);
            *reinterpret_cast<uint2*>(st + (sp ^ (uint32_t)(g * 16))) = o;
          }
        }
      }
    }
    __builtin_amdgcn_s_barrier();  // B(q)
  }
}
