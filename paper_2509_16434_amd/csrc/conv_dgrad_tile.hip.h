// Transposed 3x3 stride-2 pad-1 convolution (input gradient) for 64 gradient channels and 32 or 64
// input channels, in the LDS-image organisation of conv_tile.hip.h.
//
// The 2x2 block of input pixels (2a+py, 2b+px) - a "quad" - receives only from the four dY pixels
// (a+dyo, b+dxo), dyo, dxo in {0,1}: pixel class (py, px) uses (1+py)*(1+px) of the nine taps, nine
// tap applications per quad in all, so nothing is multiplied by zero.  A lane owns one quad: it reads
// each of the four dY pixels once per 16 channels and feeds it to every (class, tap) that uses it,
// accumulating the four pixels' CI/WGN columns in registers (64).  The weights, transposed per tap
// to [ci][co], stay in registers for the whole kernel (144).
//
// Waves of a block (512 threads): two compute waves (two 32-quad groups each per tile); two loader
// waves that copy dY bands (TQ+1 rows) into a ring of three LDS images with LDS-writing loads; four
// finishing waves (masking and writing out is the longest per-tile job, and a wave sustains only
// about one vector-memory instruction per 190 cycles) that,
// one tile behind, apply the ReLU mask of the stored activation to the staged result and write it
// out as 16-byte segments of the band (one contiguous span of the image).  The staging area is
// double-buffered, so finishing tile q-1 overlaps computing tile q; two barriers per tile order the
// three roles.  The finishing waves fetch the mask two tiles ahead with ordinary loads into two
// register sets, so their only waits are the compiler's.
//
// Fused form (C0 > 0, CI = 32): the layer below is the first convolution, whose only gradient is
// its weight gradient G0[ci][k0] = sum over pixels of dXmasked[pixel][ci] * patch[pixel][k0] with
// the pixel's 3x3 window of the C0-channel input image as patch (plus a constant 1 for the bias).
// The loaders then also copy the band's input-image rows into an LDS ring; each finishing wave takes
// a quarter of the band's pixels: it writes the masked values back into the staging area instead of to
// memory, builds the pixels' patch rows in LDS from the image rows, and contracts the two over its
// pixels with transposing LDS reads and one MFMA per 16 pixels.  The input gradient of the first
// layer's output therefore never reaches HBM.  Each block leaves one fp32 partial [CI][9*C0+1].
//
// dY pixels are 128 bytes; their 16-byte chunks are permuted by (slot >> 1) & 7, the staged pixels'
// by tile_swz_bits<CI> of the band-linear offset: lanes of one access own consecutive quads.
#pragma once
#include "conv_tile.hip.h"
#include <type_traits>

struct ConvDgradArgs {
  ImgAddr dy;                 // gradient of the layer output, images [Ho][Wo][64]
  bf16_t* dx;                 // result, images [H][W][CI] at dx + b*x_stride_b + v*x_stride_v
  const uint32_t* xbits;      // ReLU mask: sign-bit words of the stored activation, written by the forward kernels
                              // (word w of pixel p of image i at xbits[(i*H*W + p) * (CI/32) + w])
  int64_t x_stride_b, x_stride_v;
  const bf16_t* wt;           // [9][CI][64]: wt[(tap*CI + ci)*64 + co] = W[co][tap][ci]
  const bf16_t* zpage;        // 1 KiB of zeros
  int V, H, W, Ho, Wo;
  int TQ, NB, ntiles;         // quad rows per band, bands per image, nimg * NB
  // fused first-layer weight gradient only:
  ImgAddr img0;               // the first layer's input images [H0][W0][C0] (gathered through idx)
  int H0, W0;
  float* partial0;            // [gridDim.x][CI][9*C0 + 1]
  int seg_split;              // register-fused form: the loader waves share the parts of every dY row (1) or take whole rows in turn (0)
  FastDiv dv_rb0, dv_mrow;    // division by the bytes of an input-image row / of a row of mask words (register-fused form)
};

template <int CI>
struct ConvDgradShape {
  static constexpr int CO = 64, WGN = CI / 32, MT = 2, WGM = 2 / WGN, BQ = WGM * MT * 32;  // quads per tile
  static constexpr int NBUF = 3, THREADS = 512, MAXSEG = 6, MAXCH = 8, NFW = 4;  // chunks per finishing thread, finishing waves
  static int dyimg_bytes(int Wo, int TQ) { return (TQ + 1) * (Wo + 1) * 128; }
  static int stage_bytes(int W, int TQ) { return 2 * TQ * W * CI * 2; }
  static int lds_bytes(int W, int Wo, int TQ) { return NBUF * dyimg_bytes(Wo, TQ) + 2 * stage_bytes(W, TQ); }
  // fused form: image-row ring, one patch table per finishing wave, a zero chunk, the two waves' sums
  static int kp(int C0) { return 9 * C0 + 1 <= 16 ? 16 : 32; }
  static int img0_bytes(int W0, int C0, int TQ) { return (4 * TQ + 1) * W0 * C0 * 2; }
  static int fused_extra(int W, int W0, int C0, int TQ) {
    const int hp16 = (TQ * W / 2 + 15) & ~15;
    const int patch = NFW * hp16 * kp(C0) * 2, red = NFW * 32 * 32 * 4;  // the final sums reuse the patch tables
    return NBUF * img0_bytes(W0, C0, TQ) + (patch > red ? patch : red) + 16;
  }
};

__device__ __forceinline__ uint32_t dy_swz_bits(uint32_t off) { return ((off >> 8) & 7u) << 4; }

// all-ones halves for the set bits among bits (2d, 2d+1) of b: two sign-extended one-bit fields, joined by a byte permute
__device__ __forceinline__ uint32_t keep_pair(uint32_t b, int d) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_sbfe((int)b, 2 * d, 1), hi = (uint32_t)__builtin_amdgcn_sbfe((int)b, 2 * d + 1, 1);  // 0 or -1
  return __builtin_amdgcn_perm(hi, lo, 0x07060100u);  // bytes 0, 1 of lo; bytes 2, 3 of hi
}

template <int CI, int C0>
__global__ __launch_bounds__(512) void k_conv_dgrad_tile(ConvDgradArgs a) {
  static_assert(C0 == 0 || CI == 32, "the fused form is written for 32 input channels");
  typedef ConvDgradShape<CI> S;
  constexpr int CO = S::CO, CC = CO / 16, WGN = S::WGN, NBUF = S::NBUF;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int W = a.W, Wo = a.Wo, TQ = a.TQ;
  const int RP = (Wo + 1) * 128;                       // dY image row pitch
  const int dyimg_bytes = (TQ + 1) * RP;
  const int stage_bytes = 2 * TQ * W * CI * 2;
  char* const stage0 = lds + NBUF * dyimg_bytes;
  // fused form
  constexpr int K0 = 9 * C0, KP = (K0 + 1 <= 16) ? 16 : 32;
  const int RB0 = a.W0 * C0 * 2, NR0 = 4 * TQ + 1, img0_bytes = NR0 * RB0;
  const int half = TQ * W / 2;      // pixels per finishing wave
  const int hp16 = (half + 15) & ~15;  // rows of its patch table (the rows beyond `half` stay zero)
  char* const img0_ring = stage0 + 2 * stage_bytes;
  char* const patch0 = img0_ring + NBUF * img0_bytes;
  const int patch_bytes = S::NFW * hp16 * KP * 2, red_bytes = S::NFW * 32 * 32 * 4;
  char* const zero16 = patch0 + (patch_bytes > red_bytes ? patch_bytes : red_bytes);
  float* const red = reinterpret_cast<float*>(patch0);  // used after the last tile only
  if (C0 > 0 && tid < 4) reinterpret_cast<uint32_t*>(zero16)[tid] = 0u;
  if (C0 > 0) {  // the patch tables' padding rows
    const int padw = (hp16 - half) * KP / 2;  // dwords per table
    for (int i = tid; i < S::NFW * padw; i += S::THREADS) {
      const int w = i / padw, r = i - w * padw;
      reinterpret_cast<uint32_t*>(patch0 + (w * hp16 + half) * KP * 2)[r] = 0u;
    }
  }
  const int vb = xcd_block((int)blockIdx.x, (int)gridDim.x);  // this block's number in the dealing of tiles
  const int nq = (a.ntiles > vb) ? (a.ntiles - 1 - vb) / (int)gridDim.x + 1 : 0;

  // zero the right pad slot of every dY image row once
  for (int i = tid; i < NBUF * (TQ + 1) * 8; i += S::THREADS) {
    const int chunk = i & 7, row = i >> 3;
    *reinterpret_cast<uint4*>(lds + row * RP + Wo * 128 + chunk * 16) = make_uint4(0u, 0u, 0u, 0u);
  }

  if (wave == 2 || wave == 3) {
    // ------------------------------------------------------------------ loaders: image row r belongs to loader r % 2
    const int lw = wave - 2;
    const int rowbytes = Wo * 128, segs = (rowbytes + 1023) >> 10;
    const int nld0 = (img0_bytes + 1023) >> 10;  // the image rows are one contiguous span: 1 KiB pieces
    const int ni = ((TQ + 1 - lw + 1) >> 1) * segs + (C0 > 0 ? ((nld0 - lw + 1) >> 1) : 0);  // this wave's loads per band
    int goff[S::MAXSEG];
#pragma unroll
    for (int sg = 0; sg < S::MAXSEG; ++sg) {
      const uint32_t phys = sg * 1024 + lane * 16, logi = phys ^ dy_swz_bits(phys);
      goff[sg] = (sg < segs && (int)phys < rowbytes) ? (int)logi : -1;
    }
    auto issue = [&](int q) __attribute__((always_inline)) {
      const int t = vb + q * gridDim.x;
      const int img = t / a.NB, band = t - img * a.NB;
      const int oy_lo = band * TQ;
      const char* src = reinterpret_cast<const char*>(a.dy.ptr_uniform(img)) + (int64_t)oy_lo * rowbytes;
      char* dst = lds + (q % NBUF) * dyimg_bytes;
      for (int row = lw; row <= TQ; row += 2) {
        const bool inside = oy_lo + row < a.Ho;
#pragma unroll
        for (int sg = 0; sg < S::MAXSEG; ++sg)
          if (sg < segs) {
            const char* p = inside ? src + (int64_t)row * rowbytes + goff[sg] : reinterpret_cast<const char*>(a.zpage) + lane * 16;
            if (goff[sg] >= 0) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(dst + row * RP + sg * 1024), 16, 0, 0);
          }
      }
      if constexpr (C0 > 0) {
        // input-image rows 4*band*TQ - 1 ... + 4*TQ, as they are (rows outside the image: zeros); the rows
        // follow each other in memory and in LDS, so one load moves 1 KiB of them
        const int iy0 = 4 * band * TQ - 1;
        const char* isrc = reinterpret_cast<const char*>(a.img0.ptr_uniform(img)) + (int64_t)iy0 * RB0;
        char* idst = img0_ring + (q % NBUF) * img0_bytes;
        for (int j = lw; j < nld0; j += 2) {
          const int o = j * 1024 + lane * 16, iy = iy0 + o / RB0;
          const bool inside = iy >= 0 && iy < a.H0;
          const char* p = inside ? isrc + o : reinterpret_cast<const char*>(a.zpage) + lane * 16;
          if (o < img0_bytes) __builtin_amdgcn_global_load_lds(GLOBAL_AS(p), LDS_AS(idst + j * 1024), 16, 0, 0);
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
    __builtin_amdgcn_s_barrier();        // C
    __builtin_amdgcn_s_barrier();        // D
    return;
  }

  if (wave >= 4) {
    // ------------------------------------------------------------------ finishing waves
    // Unfused: the four waves share the band's chunks (thread et of 256 takes et, et+256, ...).
    // Fused: wave fw owns the pixels [fw*half, (fw+1)*half) and their chunks.
    const int et = tid - 256, fw = wave - 4;
    const int nchunk = stage_bytes >> 4;
    const int nchw = half * (CI / 8);  // chunks per finishing wave (fused)
    auto chunk_of = [&](int i) -> int { return C0 > 0 ? fw * nchw + lane + 64 * i : et + 256 * i; };
    auto chunk_mine = [&](int i) -> bool { return C0 > 0 ? lane + 64 * i < nchw : et + 256 * i < nchunk; };
    // two register sets: the mask of tile q+1 is fetched while tile q-1 is finished (two tiles of
    // mask bytes in flight per CU)
    // (the RGB fused form needs the registers for its 27-tap patches and keeps one set: one tile ahead)
    constexpr int NSET = (C0 == 3) ? 1 : 2;
    uint32_t mk[NSET][S::MAXCH];   // the word holding a chunk's eight mask bits
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
        const int c = chunk_of(i);
        // wave-uniform base + 32-bit lane offset, formed here (the empty asm keeps the compiler from
        // carrying per-chunk 64-bit addresses across the tile loop, which spills)
        uint32_t off = (uint32_t)(c >> 2) * 4u;  // four chunks (32 channels) per word
        asm volatile("" : "+v"(off));
        mk[SET][i] = (chunk_mine(i) && c < nvalid[SET]) ? *reinterpret_cast<const uint32_t*>(reinterpret_cast<const char*>(wb) + off) : 0u;
      }
    };

    // ---- fused form: patch values of this lane's pixels, the patch table, the running sums
    constexpr int PJ = 2, NV = K0 + 1, NREG = (NV + 1) / 2;
    uint32_t tp[PJ][NREG > 0 ? NREG : 1];
    int toff[PJ]; uint32_t tcol[PJ];
    f32x16_t accw;
#pragma unroll
    for (int e = 0; e < 16; ++e) accw[e] = 0.f;
    char* const patch_w = patch0 + fw * hp16 * KP * 2;
    if constexpr (C0 > 0) {
#pragma unroll
      for (int j = 0; j < PJ; ++j) {
        const int pj = lane + 64 * j, bp = fw * half + (pj < half ? pj : 0), prow = bp / W, ix = bp - prow * W;
        toff[j] = (2 * prow) * RB0 + (2 * ix - 1) * C0 * 2;                  // window corner within the band's image rows
        tcol[j] = (ix > 0 ? 1u : 0u) | 2u | (2 * ix + 1 < a.W0 ? 4u : 0u);   // window columns inside the image
      }
    }
    auto load_taps = [&](int q) __attribute__((always_inline)) {  // from the image rows of tile q (in LDS since A(q)) into registers
      if constexpr (C0 > 0) {
        const char* im = img0_ring + (q % NBUF) * img0_bytes;
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
#pragma unroll
          for (int r = 0; r < NREG; ++r) tp[j][r] = 0u;
          if (lane + 64 * j < half) {
#pragma unroll
            for (int k = 0; k < K0; ++k) {
              const int tap = k / C0, cch = k - tap * C0, u = tap / 3, v = tap - 3 * u;
              // columns outside the image read the zero chunk (no branch around the load)
              const char* src = ((tcol[j] >> v) & 1u) ? im + toff[j] + u * RB0 + (v * C0 + cch) * 2 : zero16;
              const uint32_t x = (uint32_t)*reinterpret_cast<const unsigned short*>(src);
              tp[j][k >> 1] |= x << (16 * (k & 1));
            }
            tp[j][K0 >> 1] |= 0x3F80u << (16 * (K0 & 1));  // the bias column: 1.0
          }
        }
      }
    };

    auto finish = [&](int q, auto setc) __attribute__((always_inline)) {  // tile q was loaded into set q & 1
      constexpr int SET = decltype(setc)::value;
      char* st = stage0 + (q & 1) * stage_bytes;
      // One wait for everything outstanding (this set's mask, fetched two tiles ago, and the younger
      // set's): otherwise every use of a mask register below waits for the store issued just before it.
      vm_wait<0>();
#pragma unroll
      for (int i = 0; i < S::MAXCH; ++i) {
        const int c = chunk_of(i);
        if (chunk_mine(i) && (C0 > 0 || c < nvalid[SET])) {
          const uint32_t L = (uint32_t)c * 16u, ph = L ^ tile_swz_bits<CI>(L);
          uint4 v = *reinterpret_cast<const uint4*>(st + ph);
          const uint32_t b8 = mk[SET][i] >> ((c & 3) * 8);  // this chunk's eight bits
          v.x &= keep_pair(b8, 0); v.y &= keep_pair(b8, 1); v.z &= keep_pair(b8, 2); v.w &= keep_pair(b8, 3);
          if constexpr (C0 > 0) *reinterpret_cast<uint4*>(st + ph) = v;  // chunks outside the image become zeros
          else {
            uint32_t off = L;
            asm volatile("" : "+v"(off));
            store_stream16(reinterpret_cast<bf16_t*>(reinterpret_cast<char*>(a.dx + band_off[SET]) + off), v);
          }
        }
      }
      if constexpr (C0 > 0) {
#pragma unroll
        for (int j = 0; j < PJ; ++j) {
          const int pj = lane + 64 * j;
          if (pj < half) {
#pragma unroll
            for (int r = 0; r < KP / 8; ++r) {
              uint32_t w4[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) w4[e] = (4 * r + e < NREG) ? tp[j][(4 * r + e < NREG) ? 4 * r + e : 0] : 0u;
              *reinterpret_cast<uint4*>(patch_w + pj * KP * 2 + r * 16) = make_uint4(w4[0], w4[1], w4[2], w4[3]);
            }
          }
        }
        // G0[ci][k0] += sum over this wave's pixels: both operands through transposing reads
        // Sixteen pixels further on is 1 KiB further in the staging area, which leaves the permutation
        // bits (8 and 9 of the offset) as they are: every address below is affine in the step.
        const int g = lane >> 4, r16 = lane & 15, col = 16 * (g & 1) + 4 * (r16 & 3);
        const int p = 8 * (g >> 1) + (r16 >> 2);
        const uint32_t L0 = (uint32_t)(((fw * half + p) * CI + col) * 2), L1 = L0 + 4 * CI * 2;
        const char* a0 = st + (L0 ^ tile_swz_bits<CI>(L0));
        const char* a1 = st + (L1 ^ tile_swz_bits<CI>(L1));
        const bool bz = col >= KP;  // table columns beyond KP read the zero chunk
        const char* b0 = bz ? zero16 : patch_w + (p * KP + col) * 2;
        const char* b1 = bz ? zero16 : b0 + 4 * KP * 2;
        const int bstep = bz ? 0 : 16 * KP * 2;
        int s0 = 0;
        for (; s0 + 16 <= half; s0 += 16) {
          const bf16x8_t av = lds_read_tr8_2(a0, a1);
          const bf16x8_t bv = lds_read_tr8_2(b0, b1);
          accw = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, accw, 0, 0, 0);
          a0 += 16 * CI * 2; a1 += 16 * CI * 2; b0 += bstep; b1 += bstep;
        }
        if (s0 < half) {
          // ragged last step: pixels beyond the wave's range have zero patch rows; their staged operand is
          // taken from the wave's last pixel so that nothing outside the range is read
          const int pa = min(s0 + p, half - 1), pb = min(s0 + p + 4, half - 1);
          const uint32_t M0 = (uint32_t)(((fw * half + pa) * CI + col) * 2), M1 = (uint32_t)(((fw * half + pb) * CI + col) * 2);
          const bf16x8_t av = lds_read_tr8_2(st + (M0 ^ tile_swz_bits<CI>(M0)), st + (M1 ^ tile_swz_bits<CI>(M1)));
          const bf16x8_t bv = lds_read_tr8_2(b0, b1);
          accw = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, accw, 0, 0, 0);
        }
      }
    };
    typedef std::integral_constant<int, 0> set0;
    typedef std::integral_constant<int, 1> set1;
    auto step = [&](int q, auto par) __attribute__((always_inline)) {  // q & 1 == par
      constexpr int P = decltype(par)::value;
      typedef std::integral_constant<int, 1 - P> other;
      __builtin_amdgcn_s_barrier();  // A(q)
      if constexpr (NSET == 2) {
        if (q > 0) {
          finish(q - 1, other());
          if (q + 1 < nq) load_mask(q + 1, other());
        }
      } else {
        if (q > 0) finish(q - 1, set0());
        load_mask(q, set0());
      }
      load_taps(q);
      __builtin_amdgcn_s_barrier();  // B(q): tile q is staged
    };
    if constexpr (NSET == 2) {
      if (nq > 0) load_mask(0, set0());
      if (nq > 1) load_mask(1, set1());
    }
    for (int q = 0; q < nq; q += 2) {
      step(q, set0());
      if (q + 1 < nq) step(q + 1, set1());
    }
    if (nq > 0) {
      if constexpr (NSET == 2) { if ((nq - 1) & 1) finish(nq - 1, set1()); else finish(nq - 1, set0()); }
      else finish(nq - 1, set0());
    }
    __builtin_amdgcn_s_barrier();    // C: every finishing wave is done with its patch table
    if constexpr (C0 > 0) {
      // accw[e] = G0[ci][k0] with k0 = lane % 32, ci = (e/4)*8 + (lane/32)*4 + e%4
#pragma unroll
      for (int e = 0; e < 16; ++e) red[fw * 1024 + ((e >> 2) * 8 + (lane >> 5) * 4 + (e & 3)) * 32 + (lane & 31)] = accw[e];
    }
    __builtin_amdgcn_s_barrier();    // D
    if constexpr (C0 > 0) {
      if (fw == 0) {
        float* P = a.partial0 + (int64_t)blockIdx.x * CI * NV;
        for (int i = lane; i < CI * NV; i += 64) {
          const int ci = i / NV, k = i - ci * NV;
          P[i] = (red[ci * 32 + k] + red[1024 + ci * 32 + k]) + (red[2048 + ci * 32 + k] + red[3072 + ci * 32 + k]);
        }
      }
    }
    return;
  }

  // -------------------------------------------------------------------- compute waves
  const int l32 = lane & 31, h = lane >> 5;
  constexpr int MT = S::MT;
  const int wm = wave / WGN, wn = wave % WGN;
  // weights: lane (column ci = wn*32 + l32, 8 co at cc*16 + h*8) of tap s
  bf16x8_t wr[9][CC];
#pragma unroll
  for (int s = 0; s < 9; ++s)
#pragma unroll
    for (int cc = 0; cc < CC; ++cc)
      wr[s][cc] = *reinterpret_cast<const bf16x8_t*>(a.wt + ((int64_t)s * CI + wn * 32 + l32) * CO + cc * 16 + h * 8);

  for (int q = 0; q < nq; ++q) {
    const int t = vb + q * gridDim.x;
    const int band = t % a.NB;
    __builtin_amdgcn_s_barrier();  // A(q): band q is in LDS, staging buffer q&1 is free
    char* st = stage0 + (q & 1) * stage_bytes;
    const int rows_here = a.H - 2 * band * TQ;  // image rows left from the band's first row
#pragma unroll 1
    for (int mt = 0; mt < MT; ++mt) {
      // this lane's quad of the group (lanes beyond the band work on quad 0 and store nothing);
      // recomputed per tile: registers are scarcer here than ALU cycles
      const int qi = (wm * MT + mt) * 32 + l32;
      const bool in_band = qi < TQ * Wo;
      const int al = in_band ? qi / Wo : 0, b = in_band ? qi - al * Wo : 0;
      const char* img_s = lds + (q % NBUF) * dyimg_bytes + al * RP + b * 128;
      uint32_t hx[2];
#pragma unroll
      for (int dxo = 0; dxo < 2; ++dxo) hx[dxo] = (uint32_t)(h * 16) ^ dy_swz_bits((uint32_t)((b + dxo) * 128));
      f32x16_t acc[4];
#pragma unroll
      for (int c = 0; c < 4; ++c)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
      // The four dY pixels are fetched one pixel (all its channel chunks) ahead of the MFMAs that use
      // them, so that the LDS latency of a lone wave per SIMD hides behind 4 to 16 MFMAs.
      bf16x8_t av[2][CC];
      auto fetch = [&](int pi, bf16x8_t (&dst)[CC]) __attribute__((always_inline)) {
        const int dyo = pi >> 1, dxo = pi & 1;
#pragma unroll
        for (int cc = 0; cc < CC; ++cc)
          dst[cc] = *reinterpret_cast<const bf16x8_t*>(img_s + dyo * RP + dxo * 128 + ((uint32_t)(cc * 32) ^ hx[dxo]));
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
  __builtin_amdgcn_s_barrier();    // C
  __builtin_amdgcn_s_barrier();    // D
}
