// Bandwidth-bound and elementwise kernels of the learner: buffer append, GAE scan, minibatch
// permutation, first-layer convolution (K = 9 or 27: too thin for MFMA), losses, Adam and
// weight re-packing.
#pragma once
#include "common.hip.h"
#include "gemm.hip.h"

// The per-step scalars of a rollout slab: proprio (-> bf16), action, log-prob, value, reward, done.
struct ScalarWrite {
  int N, P, A;
  const float *proprio, *action, *logp, *value, *reward;
  const uint8_t* done;
  bf16_t* o_proprio;
  float *o_action, *o_logp, *o_value, *o_reward;
  uint8_t* o_done;
};
__device__ __forceinline__ void write_scalars(int64_t i, const ScalarWrite& w) {
  if (i < (int64_t)w.N * w.P) w.o_proprio[i] = f2bf(w.proprio[i]);
  if (w.action && i < (int64_t)w.N * w.A) w.o_action[i] = w.action[i];
  if (i < w.N) {
    if (w.logp) w.o_logp[i] = w.logp[i];
    if (w.value) w.o_value[i] = w.value[i];
    if (w.reward) w.o_reward[i] = w.reward[i];
    if (w.done) w.o_done[i] = w.done[i];
  }
}

// ---------------------------------------------------------------- buffer append
// One step's images [N][V][C][HW] (fp32 or bf16) -> bf16 channel-last [N][V][HW][C] at the
// step's slab.  Each thread converts 8 consecutive pixels of one (n, v) image; the blocks behind
// the last image block write the slab's scalars (one launch per rollout step).
template <typename InT>
__global__ void k_write_obs(const InT* __restrict__ src, bf16_t* __restrict__ dst, int64_t n_img, int C, int HW, int obs_blocks, ScalarWrite sw) {
  const int groups = (HW + 7) / 8;
  if ((int)blockIdx.x >= obs_blocks) {  // the blocks behind the images write the slab's scalars
    write_scalars((int64_t)((int)blockIdx.x - obs_blocks) * blockDim.x + threadIdx.x, sw);
    return;
  }
  int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (gid >= n_img * groups) return;
  int64_t img = gid / groups;
  int p0 = (int)(gid - img * groups) * 8;
  const InT* s = src + img * (int64_t)C * HW;
  bf16_t* d = dst + img * (int64_t)C * HW;
  auto cvt = [](InT x) -> bf16_t {
    if constexpr (sizeof(InT) == 4) return f2bf((float)x); else return (bf16_t)x;
  };
  if (C == 1 && p0 + 8 <= HW) {
    bf16_t o[8];
    if constexpr (sizeof(InT) == 4) {
      const float4* s4 = reinterpret_cast<const float4*>(s + p0);
      float4 a = s4[0], b = s4[1];
      o[0] = f2bf(a.x); o[1] = f2bf(a.y); o[2] = f2bf(a.z); o[3] = f2bf(a.w);
      o[4] = f2bf(b.x); o[5] = f2bf(b.y); o[6] = f2bf(b.z); o[7] = f2bf(b.w);
      *reinterpret_cast<uint4*>(d + p0) = *reinterpret_cast<uint4*>(o);
    } else {
      *reinterpret_cast<uint4*>(d + p0) = *reinterpret_cast<const uint4*>(s + p0);
    }
    return;
  }
  if (C == 3 && p0 + 8 <= HW && (HW & 7) == 0) {
    // planar RGB -> interleaved: three 8-pixel runs in (16 or 32 bytes each), 24 bf16 = three 16-byte stores out
    bf16_t in[3][8];
#pragma unroll
    for (int c = 0; c < 3; ++c) {
      if constexpr (sizeof(InT) == 4) {
        const float4* s4 = reinterpret_cast<const float4*>(s + (int64_t)c * HW + p0);
        const float4 a = s4[0], b = s4[1];
        in[c][0] = f2bf(a.x); in[c][1] = f2bf(a.y); in[c][2] = f2bf(a.z); in[c][3] = f2bf(a.w);
        in[c][4] = f2bf(b.x); in[c][5] = f2bf(b.y); in[c][6] = f2bf(b.z); in[c][7] = f2bf(b.w);
      } else {
        *reinterpret_cast<uint4*>(in[c]) = *reinterpret_cast<const uint4*>(s + (int64_t)c * HW + p0);
      }
    }
    bf16_t o[24];
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int c = 0; c < 3; ++c) o[j * 3 + c] = in[c][j];
    uint4* d4 = reinterpret_cast<uint4*>(d + (int64_t)p0 * 3);
#pragma unroll
    for (int q = 0; q < 3; ++q) d4[q] = reinterpret_cast<const uint4*>(o)[q];
    return;
  }
  for (int j = 0; j < 8; ++j) {
    int p = p0 + j;
    if (p >= HW) break;
    for (int c = 0; c < C; ++c) d[(int64_t)p * C + c] = cvt(s[(int64_t)c * HW + p]);
  }
}

// Inverse layout change of k_write_obs (no conversion): channel-last -> [img][C][HW].
__global__ void k_read_obs(const bf16_t* __restrict__ src, bf16_t* __restrict__ dst, int64_t n_img, int C, int HW) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t per = (int64_t)C * HW;
  if (i >= n_img * per) return;
  int64_t img = i / per; int r = (int)(i - img * per), c = r / HW, p = r - c * HW;
  dst[i] = src[img * per + (int64_t)p * C + c];
}


// ---------------------------------------------------------------- GAE
// One thread per environment, reverse scan over time held in registers; at every t the wave reads/writes
// N-contiguous rows.  The scan itself is a dependent chain of a few flops per step, the loads are not: the
// rewards, values and done flags of up to TC steps are all requested before the first of them is used, so an
// environment pays one memory round trip per TC steps instead of one per step (loads and stores return in
// order on this hardware: a load issued behind a store waits for it).
template <int TC>
__global__ __launch_bounds__(64) void k_gae(int T, int N, const float* __restrict__ reward, const uint8_t* __restrict__ done,
                                            const float* __restrict__ value, const float* __restrict__ last_value, float gamma, float lambda,
                                            float* __restrict__ adv, float* __restrict__ ret) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float next_v = last_value[n], next_a = 0.f;
  for (int t1 = T; t1 > 0; t1 -= TC) {  // steps [t0, t1), last chunk first
    const int t0 = t1 > TC ? t1 - TC : 0, cnt = t1 - t0;
    // No branch between the loads (a slot beyond the chunk re-reads the chunk's last step): the compiler
    // drains every outstanding load at a branch target, which would put the round trips back in a row.
    float r[TC], v[TC];
    uint8_t d[TC];
#pragma unroll
    for (int j = 0; j < TC; ++j) {
      const int64_t i = (int64_t)(t0 + (j < cnt ? j : cnt - 1)) * N + n;
      r[j] = reward[i]; v[j] = value[i]; d[j] = done[i];
    }
    asm volatile("" ::: "memory");  // every load above is issued before the first store below (the scheduler would sink them to their uses)
    // Slots beyond the chunk come first in this order; they leave the running pair untouched and write the
    // chunk's last step, which that step's own turn then overwrites (same thread, same address: in order).
#pragma unroll
    for (int j = TC - 1; j >= 0; --j) {
      const bool live = j < cnt;
      const int64_t i = (int64_t)(t0 + (live ? j : cnt - 1)) * N + n;
      const float nt = d[j] ? 0.f : 1.f;
      const float delta = r[j] + gamma * next_v * nt - v[j];
      const float a = delta + gamma * lambda * nt * next_a;
      adv[i] = a; ret[i] = a + v[j];
      next_a = live ? a : next_a; next_v = live ? v[j] : next_v;
    }
  }
}

// ---------------------------------------------------------------- permutation
// perm = indices sorted by (key_i, i), key_i = i-th output of a SplitMix64 generator whose
// state is derived from (seed, update, epoch).  Keys are uniform, so a bucket pass on the top
// bits followed by an exact rank inside each (small) bucket gives the sorted order without
// a general sort; the result does not depend on the order of the atomic scatter.
__host__ __device__ __forceinline__ uint64_t sm64_mix(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
__host__ __device__ __forceinline__ uint64_t perm_stream(uint64_t seed, uint64_t update, uint64_t epoch) {
  const uint64_t G = 0x9E3779B97F4A7C15ULL;
  uint64_t s = sm64_mix(seed + G);
  s = sm64_mix(s ^ (update + G));
  s = sm64_mix(s ^ (epoch + G));
  return s;
}
__device__ __forceinline__ uint64_t perm_key(uint64_t stream, uint64_t i) {
  return sm64_mix(stream + (i + 1) * 0x9E3779B97F4A7C15ULL);
}
__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
// The kernels below work on up to PERM_BATCH permutations (the epochs of one update) at once: blockIdx.y is the slot,
// with its own generator state, histogram + cursor (2*nb words), bucket starts (nb), scratch and result (S each).
#define PERM_BATCH 8
struct PermStreams { uint64_t s[PERM_BATCH]; };
__global__ void k_perm_hist(PermStreams ps, int S, int shift, int nb, int32_t* __restrict__ hist_all) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S) return;
  const uint64_t stream = ps.s[blockIdx.y];
  int32_t* hist = hist_all + (int64_t)blockIdx.y * 2 * nb;
  int b = shift >= 64 ? 0 : (int)(perm_key(stream, (uint64_t)i) >> shift);
  atomicAdd(&hist[b], 1);
}
// exclusive scan of hist[nb] into start[nb]; one block of 1024 threads per slot
__global__ void k_perm_scan(const int32_t* __restrict__ hist_all, int32_t* __restrict__ start_all, int nb) {
  __shared__ int32_t part[1024];
  const int32_t* hist = hist_all + (int64_t)blockIdx.y * 2 * nb;
  int32_t* start = start_all + (int64_t)blockIdx.y * nb;
  int tid = threadIdx.x, per = (nb + 1023) / 1024, b0 = tid * per, s = 0;
  for (int j = 0; j < per; ++j) if (b0 + j < nb) s += hist[b0 + j];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) { int run = 0; for (int j = 0; j < 1024; ++j) { int v = part[j]; part[j] = run; run += v; } }
  __syncthreads();
  int run = part[tid];
  for (int j = 0; j < per; ++j) if (b0 + j < nb) { start[b0 + j] = run; run += hist[b0 + j]; }
}
__global__ void k_perm_scatter(PermStreams ps, int S, int shift, int nb, const int32_t* __restrict__ start_all,
                               int32_t* __restrict__ hist_all, int32_t* __restrict__ tmp_all) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S) return;
  const uint64_t stream = ps.s[blockIdx.y];
  const int32_t* start = start_all + (int64_t)blockIdx.y * nb;
  int32_t* cursor = hist_all + (int64_t)blockIdx.y * 2 * nb + nb;
  int32_t* tmp = tmp_all + (int64_t)blockIdx.y * S;
  int b = shift >= 64 ? 0 : (int)(perm_key(stream, (uint64_t)i) >> shift);
  int pos = start[b] + atomicAdd(&cursor[b], 1);
  tmp[pos] = i;
}
__global__ void k_perm_rank(PermStreams ps, int S, int shift, int nb, const int32_t* __restrict__ start_all,
                            const int32_t* __restrict__ hist_all, const int32_t* __restrict__ tmp_all, int32_t* __restrict__ perm_all) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= S) return;
  const uint64_t stream = ps.s[blockIdx.y];
  const int32_t* start = start_all + (int64_t)blockIdx.y * nb;
  const int32_t* hist = hist_all + (int64_t)blockIdx.y * 2 * nb;
  const int32_t* tmp = tmp_all + (int64_t)blockIdx.y * S;
  int32_t* perm = perm_all + (int64_t)blockIdx.y * S;
  int i = tmp[p];
  uint64_t key = perm_key(stream, (uint64_t)i);
  int b = shift >= 64 ? 0 : (int)(key >> shift);
  int beg = start[b], cnt = hist[b], rank = 0;
  for (int q = beg; q < beg + cnt; ++q) {
    int j = tmp[q];
    uint64_t kj = perm_key(stream, (uint64_t)j);
    rank += (kj < key || (kj == key && j < i)) ? 1 : 0;
  }
  perm[beg + rank] = i;
}

// ---------------------------------------------------------------- first convolution
// 3x3 stride-2 pad-1 convolution of a 1- or 3-channel image read straight from the rollout buffer
// through the minibatch index (the gather is fused into the loader).  K = 9*CIN (9 or 27) is padded
// to 16 / 32 and fed to the matrix cores: one 32x32x16 MFMA produces 32 pixels x 32 channels.
// The work is bound by the 64 B/pixel (Cout = 32) of activation traffic, not by arithmetic.

// flat output-pixel index -> (img, oy, ox), then stepped without divisions
struct PixCursor {
  int img, oy, ox;
  __device__ __forceinline__ void init(int64_t m, int Ho, int Wo) {
    const int hw = Ho * Wo;
    img = (int)(m / hw);
    const int q = (int)(m - (int64_t)img * hw);
    oy = q / Wo; ox = q - oy * Wo;
  }
  __device__ __forceinline__ void advance(int d, int Ho, int Wo) {
    ox += d;
    while (ox >= Wo) { ox -= Wo; ++oy; }
    while (oy >= Ho) { oy -= Ho; ++img; }
  }
};

__device__ __forceinline__ bf16x8_t pack8(const bf16_t (&x)[8]) {
  uint4 u;
  u.x = (uint32_t)x[0] | ((uint32_t)x[1] << 16); u.y = (uint32_t)x[2] | ((uint32_t)x[3] << 16);
  u.z = (uint32_t)x[4] | ((uint32_t)x[5] << 16); u.w = (uint32_t)x[6] | ((uint32_t)x[7] << 16);
  return __builtin_bit_cast(bf16x8_t, u);
}

// Forward.  A wave handles TPW tiles of 32 consecutive output pixels.  MFMA operands: weights
// [co][k] first (lane: co = lane%32, k = (lane/32)*8..+7), patches second (lane: pixel = lane%32),
// so a lane ends up with 4 groups of 4 consecutive channels of ONE pixel; bias + ReLU, pack, stage
// in wave-private LDS, and leave as 16-byte pieces of the contiguous [pixel][Cout] output.
template <int CIN, int TPW, bool RELU = true>
__global__ __launch_bounds__(256) void k_conv1_fwd(ImgAddr in, int n_img, int H, int W, int Ho, int Wo, int Cout,
                                                   const bf16_t* __restrict__ Wb, const float* __restrict__ bias,
                                                   bf16_t* __restrict__ out) {
  constexpr int K = 9 * CIN, KS = (K + 15) / 16;
  __shared__ __attribute__((aligned(16))) bf16_t stage[4][32 * 72];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int64_t M = (int64_t)n_img * Ho * Wo;
  const int NJ = (Cout + 31) / 32, SP = Cout + 8;
  bf16x8_t bw[2][KS];
  float bs[2][16];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn) {
    const int co = jn * 32 + l32;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16_t t[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) { const int k = ks * 16 + h * 8 + j; t[j] = (k < K && co < Cout) ? Wb[co * K + k] : (bf16_t)0; }
      bw[jn][ks] = pack8(t);
    }
#pragma unroll
    for (int e = 0; e < 16; ++e) { const int c2 = jn * 32 + (e >> 2) * 8 + h * 4 + (e & 3); bs[jn][e] = c2 < Cout ? bias[c2] : 0.f; }
  }
  // this lane's eight patch entries k = ks*16 + h*8 + j as (row tap u, element offset v*CIN + c)
  const int64_t mw = (int64_t)(blockIdx.x * 4 + wave) * TPW * 32;  // first pixel of this wave
  PixCursor pc; pc.init((mw + l32 < M) ? mw + l32 : 0, Ho, Wo);
  int pimg = pc.img;
  const bf16_t* p = in.ptr(pimg);
  for (int t = 0; t < TPW; ++t) {
    const int64_t m0 = mw + t * 32;
    const int64_t m = m0 + l32;
    const bool valid = m < M;
    const int iyb = 2 * pc.oy - 1, ixb = 2 * pc.ox - 1;
    const bool rok[3] = {iyb >= 0, true, iyb + 2 < H};
    const bool cok[3] = {ixb >= 0, true, ixb + 2 < W};
    const bf16_t* pb = p + (iyb * W + ixb) * CIN;
    bf16x8_t a[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16_t x[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        // both halves' k are compile-time; pick by h
        constexpr int dummy = 0; (void)dummy;
        const int k0 = ks * 16 + j, k1 = ks * 16 + 8 + j;
        const int t0 = k0 / CIN, c0 = k0 - t0 * CIN, u0 = t0 / 3, v0 = t0 - 3 * u0;
        const int t1 = k1 / CIN, c1 = k1 - t1 * CIN, u1 = t1 / 3, v1 = t1 - 3 * u1;
        const bool in0 = k0 < K, in1 = k1 < K;
        const bool ok0 = in0 && rok[in0 ? u0 : 0] && cok[in0 ? v0 : 0];
        const bool ok1 = in1 && rok[in1 ? u1 : 0] && cok[in1 ? v1 : 0];
        const int off0 = in0 ? (u0 * W + v0) * CIN + c0 : 0, off1 = in1 ? (u1 * W + v1) * CIN + c1 : 0;
        const bool ok = valid && (h ? ok1 : ok0);
        x[j] = ok ? pb[h ? off1 : off0] : (bf16_t)0;
      }
      a[ks] = pack8(x);
    }
    __syncthreads();  // previous tile's staging reads are done
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
      if (jn >= NJ) break;
      f32x16_t acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw[jn][ks], a[ks], acc, 0, 0, 0);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int cl = jn * 32 + g * 8 + h * 4;
        if (cl < Cout) {
          uint2 o;
          const float lo = RELU ? 0.f : -3.0e38f;  // without the ReLU (a layer normalisation follows) the sums pass as they are
          o.x = pack2bf(fmaxf(acc[g * 4] + bs[jn][g * 4], lo), fmaxf(acc[g * 4 + 1] + bs[jn][g * 4 + 1], lo));
          o.y = pack2bf(fmaxf(acc[g * 4 + 2] + bs[jn][g * 4 + 2], lo), fmaxf(acc[g * 4 + 3] + bs[jn][g * 4 + 3], lo));
          *reinterpret_cast<uint2*>(&stage[wave][l32 * SP + cl]) = o;
        }
      }
    }
    __syncthreads();
    const int cpr = Cout >> 3;  // 16-byte chunks per pixel
    for (int ch = lane; ch < 32 * cpr; ch += 64) {
      const int r = ch / cpr, cg = ch - r * cpr;
      if (m0 + r < M) *reinterpret_cast<uint4*>(out + (m0 + r) * Cout + cg * 8) = *reinterpret_cast<const uint4*>(&stage[wave][r * SP + cg * 8]);
    }
    if (t + 1 < TPW && m + 32 < M) {
      pc.advance(32, Ho, Wo);
      if (pc.img != pimg) { pimg = pc.img; p = in.ptr(pimg); }
    }
  }
}

// Weight/bias gradient: dW[co][k] = sum_m dY[m][co] * x[m][k], db[co] = sum_m dY[m][co] (k = K is a
// column of ones).  The contraction runs over pixels, 16 per MFMA: first operand dY^T (lane: co =
// lane%32, 8 consecutive pixels), second operand the patches (lane: k = lane%32, the same 8 pixels).
// A block walks its pixel range (waves interleaved in steps of 16 pixels), sums the four wave
// accumulators through LDS and writes one partial per block (summed later in block order).
template <int CIN>
__global__ __launch_bounds__(256) void k_conv1_wgrad(ImgAddr in, int n_img, int H, int W, int Ho, int Wo, int Cout,
                                                     const bf16_t* __restrict__ dy, int pixels_per_block,
                                                     float* __restrict__ partial) {
  constexpr int K = 9 * CIN, KP1 = K + 1;
  __shared__ float wsum[4][64 * 32];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int NJ = (Cout + 31) / 32;
  const int64_t M = (int64_t)n_img * Ho * Wo;
  const int64_t mbeg = (int64_t)blockIdx.x * pixels_per_block;
  const int64_t mend = (mbeg + pixels_per_block < M) ? mbeg + pixels_per_block : M;
  // this lane's patch column
  const int tap = l32 / CIN, cch = l32 - tap * CIN, u = tap / 3, v = tap - 3 * u;
  const bool kcol = l32 < K, kone = l32 == K;
  f32x16_t acc[2];
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[jn][e] = 0.f;
  int64_t mb = mbeg + wave * 16 + h * 8;  // first of this lane's 8 pixels
  PixCursor pc; pc.init(mb < mend ? mb : 0, Ho, Wo);
  const bf16_t* p = in.ptr(mb < mend ? pc.img : 0);
  int pimg = pc.img;
  for (; mb - h * 8 < mend; mb += 64) {
    bf16_t xs[8], ds[2][8];
    PixCursor q = pc;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const bool ok = mb + j < mend;
      bf16_t xv = 0;
      if (ok && kone) xv = 0x3F80;  // 1.0
      if (ok && kcol) {
        const bf16_t* pj = (q.img == pimg) ? p : in.ptr(q.img);
        const int iy = 2 * q.oy - 1 + u, ix = 2 * q.ox - 1 + v;
        if ((unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W) xv = pj[(iy * W + ix) * CIN + cch];
      }
      xs[j] = xv;
#pragma unroll
      for (int jn = 0; jn < 2; ++jn) {
        const int co = jn * 32 + l32;
        ds[jn][j] = (ok && co < Cout) ? dy[(mb + j) * Cout + co] : (bf16_t)0;
      }
      q.advance(1, Ho, Wo);
    }
    const bf16x8_t xb = pack8(xs);
#pragma unroll
    for (int jn = 0; jn < 2; ++jn) {
      if (jn >= NJ) break;
      acc[jn] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pack8(ds[jn]), xb, acc[jn], 0, 0, 0);
    }
    if (mb + 64 < mend) {
      pc.advance(64, Ho, Wo);
      if (pc.img != pimg) { pimg = pc.img; p = in.ptr(pimg); }
    }
  }
  // acc[jn][g*4+q] = D[co = jn*32 + g*8 + h*4 + q][k = l32]
#pragma unroll
  for (int jn = 0; jn < 2; ++jn)
#pragma unroll
    for (int e = 0; e < 16; ++e) wsum[wave][(jn * 32 + (e >> 2) * 8 + h * 4 + (e & 3)) * 32 + l32] = acc[jn][e];
  __syncthreads();
  float* P = partial + (int64_t)blockIdx.x * Cout * KP1;
  for (int i = tid; i < Cout * KP1; i += 256) {
    const int co = i / KP1, k = i - co * KP1, s = co * 32 + k;
    P[i] = (wsum[0][s] + wsum[1][s]) + (wsum[2][s] + wsum[3][s]);
  }
}

// ---------------------------------------------------------------- gather of small per-sample data
// proprio (bf16 in the buffer) -> columns [col0, col0+P) of the feature matrix.
__global__ void k_gather_proprio(const bf16_t* __restrict__ proprio, const int32_t* __restrict__ idx, int B, int P,
                                 bf16_t* __restrict__ feat, int64_t ld, int col0) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)B * P) return;
  int b = (int)(i / P), j = (int)(i - (int64_t)b * P);
  int64_t s = idx ? idx[b] : b;
  feat[(int64_t)b * ld + col0 + j] = proprio[s * P + j];
}

// The auxiliary MLP head's slice of the loss gradient: columns [col0, col0 + X) of the head-gradient rows
// dhead [B][32] move to columns [0, X) of daux [B][32], the rest of a daux row is zero.
__global__ void k_aux_cols(int B, int col0, int X, const bf16_t* __restrict__ dhead, bf16_t* __restrict__ daux) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)B * 32) return;
  const int j = (int)(i & 31);
  daux[i] = j < X ? dhead[(i - j) + col0 + j] : (bf16_t)0;
}
// a[i] = bf16(a[i] + b[i]): two gradient contributions to one stored activation (eight elements per thread)
__global__ void k_add_bf16(int64_t n8, bf16_t* __restrict__ a, const bf16_t* __restrict__ b) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n8) return;
  uint4 x = reinterpret_cast<const uint4*>(a)[i];
  const uint4 y = reinterpret_cast<const uint4*>(b)[i];
  auto add2 = [](uint32_t u, uint32_t v) { return pack2bf(bf2f((bf16_t)(u & 0xffffu)) + bf2f((bf16_t)(v & 0xffffu)), bf2f((bf16_t)(u >> 16)) + bf2f((bf16_t)(v >> 16))); };
  x.x = add2(x.x, y.x); x.y = add2(x.y, y.y); x.z = add2(x.z, y.z); x.w = add2(x.w, y.w);
  reinterpret_cast<uint4*>(a)[i] = x;
}

// ---------------------------------------------------------------- losses
#define LOSS_NSTAT 8  // pi, v, kl, clipfrac sums; slots 4..7 unused
#define HEAD_LD 32    // row stride of the head output / head gradient matrices
#define LOSS_BLOCK 64  // samples (threads) per block of the loss kernels: one wave, so that a minibatch spreads over many CUs

// Reward and termination flag of one step, which arrive after the simulators have stepped.
__global__ void k_write_outcome(int N, const float* __restrict__ reward, const uint8_t* __restrict__ done, float* __restrict__ o_reward,
                                uint8_t* __restrict__ o_done) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < N) { o_reward[i] = reward[i]; o_done[i] = done[i]; }
}

// ---------------------------------------------------------------- policy step
// Sampling of the collection loop's action (Algorithm 2: actions from the stacked observations)
// from the head outputs of n samples (row: A means, then the value):
//   a_j = mu_j + exp(logstd_j) * xi_j,  logp = sum_j [-z_j^2/2 - logstd_j - ln(2 pi)/2],  z = (a - mu)/sigma
// z is formed from the rounded action, with the arithmetic of the loss kernels, so that the loss
// sees ratio 1 on fresh data.  One thread per sample; results go to the rollout slab (o_*) and,
// where given, to the caller's arrays (c_*).
__global__ void k_act_sample(int n, int A, const float* __restrict__ headout, const float* __restrict__ logstd, const float* __restrict__ noise,
                             float* __restrict__ o_action, float* __restrict__ o_logp, float* __restrict__ o_value,
                             float* __restrict__ c_action, float* __restrict__ c_logp, float* __restrict__ c_value) {
  const int s = blockIdx.x * blockDim.x + threadIdx.x;
  if (s >= n) return;
  const float* o = headout + (int64_t)s * HEAD_LD;
  float logp = 0.f;
  for (int j = 0; j < A; ++j) {
    const float ls = logstd[j], sg = expf(ls), sig_inv = __expf(-ls), mu = o[j];
    const float a = mu + sg * noise[(int64_t)s * A + j];
    const float zz = (a - mu) * sig_inv;
    logp += -0.5f * zz * zz - ls - 0.91893853320467274178f;
    o_action[(int64_t)s * A + j] = a;
    if (c_action) c_action[(int64_t)s * A + j] = a;
  }
  const float v = o[A];
  o_logp[s] = logp; o_value[s] = v;
  if (c_logp) c_logp[s] = logp;
  if (c_value) c_value[s] = v;
}

// Per-sample inputs of the losses (rollout arrays indexed by the gathered sample number).
struct LossData {
  int Bfull, A;
  const float* logstd;
  const int32_t* idx;
  const float *action, *logp_old, *v_old, *adv, *ret;
  float clip_eps, vclip_eps, vf_coef;
  int aux_dim;      // distillation: the last aux_dim columns are the auxiliary output (0: none)
  float aux_coef;   // and their error's weight
};

// Clipped-surrogate PPO loss of one sample (number s of the rollout) of a minibatch of `Bfull`:
//   logp = sum_j [-z_j^2/2 - logstd_j - ln(2 pi)/2], z = (a - mu)/sigma; rho = exp(logp - logp_old)
//   L_pi = -mean min(rho A, clip(rho, 1-eps, 1+eps) A);  L_V = mean (V-R)^2 or its clipped max form
// o: the head's output row (means, then the value).  Leaves the gradient row dL/dmu_0..A-1, dL/dV
// (bf16 pairs, zero padded to 32 columns) in pk, this sample's terms of the four statistics in st and
// of dL/dlogstd in dls.
// The rollout's values of one sample, gathered without a branch in between, so that every load is
// issued before the first one is used: one memory latency, not A of them.
struct LossSample { float act[32], lpo, adv, ret, vo; };
__device__ __forceinline__ LossSample loss_gather(const LossData& L, int64_t s, bool ppo) {
  LossSample g;
  const int A = L.A;
#pragma unroll
  for (int j = 0; j < 32; ++j) g.act[j] = L.action[s * A + (j < A ? j : A - 1)];
  g.lpo = ppo ? L.logp_old[s] : 0.f; g.adv = ppo ? L.adv[s] : 0.f; g.ret = ppo ? L.ret[s] : 0.f; g.vo = ppo ? L.v_old[s] : 0.f;
  return g;
}
__device__ __forceinline__ void ppo_loss_sample(const LossData& L, const float* sig_inv, const float* ls, const LossSample& smp, const float (&o)[HEAD_LD],
                                                uint32_t (&pk)[16], float (&st)[4], float (&dls)[32]) {
  const int A = L.A;
  const float invB = 1.f / (float)L.Bfull;
  const float (&act)[32] = smp.act;
  const float lpo = smp.lpo, a = smp.adv, r = smp.ret, vo = smp.vo;
  float z[32];
  float logp = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float zz = (act[j] - o[j]) * sig_inv[j < A ? j : 0];
    z[j] = j < A ? zz : 0.f;
    logp += j < A ? -0.5f * zz * zz - ls[j < A ? j : 0] - 0.91893853320467274178f : 0.f;
  }
  const float lr = logp - lpo, rho = expf(lr);
  const float rc = fminf(fmaxf(rho, 1.f - L.clip_eps), 1.f + L.clip_eps);
  const float s1 = rho * a, s2 = rc * a;
  st[0] = -fminf(s1, s2);
  const float dlogp = (s1 <= s2) ? -invB * a * rho : 0.f;
  st[2] = (rho - 1.f) - lr;
  st[3] = fabsf(rho - 1.f) > L.clip_eps ? 1.f : 0.f;
  float v = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j) v = (j == A) ? o[j] : v;  // the value head's column (register array: no dynamic index)
  const float err = v - r;
  float dv;
  if (L.vclip_eps > 0.f) {
    const float d = v - vo, dc = fminf(fmaxf(d, -L.vclip_eps), L.vclip_eps), errc = vo + dc - r;
    if (errc * errc > err * err) { st[1] = errc * errc; dv = (d >= -L.vclip_eps && d <= L.vclip_eps) ? 2.f * errc : 0.f; }
    else { st[1] = err * err; dv = 2.f * err; }
  } else { st[1] = err * err; dv = 2.f * err; }
#pragma unroll
  for (int j = 0; j < 32; j += 2) {
    float g0 = 0.f, g1 = 0.f;
    if (j < A) g0 = dlogp * z[j] * sig_inv[j];
    else if (j == A) g0 = L.vf_coef * invB * dv;
    if (j + 1 < A) g1 = dlogp * z[j + 1] * sig_inv[j + 1];
    else if (j + 1 == A) g1 = L.vf_coef * invB * dv;
    pk[j >> 1] = pack2bf(g0, g1);
  }
#pragma unroll
  for (int j = 0; j < 32; ++j) dls[j] = j < A ? dlogp * (z[j] * z[j] - 1.f) : 0.f;
}

// Distillation loss of one sample: sums over the action columns (st[0]) and over the auxiliary columns (st[1]) of
// (pred - teacher)^2, scaled later; the gradient carries the scales 1/(B (A-X)) and aux_coef/(B X).
__device__ __forceinline__ void mse_loss_sample(const LossData& L, const LossSample& smp, const float (&o)[HEAD_LD], uint32_t (&pk)[16], float (&st)[4]) {
  const int A = L.A, Aa = A - L.aux_dim;
  const float sa = 1.f / ((float)L.Bfull * (float)Aa), sx = L.aux_dim > 0 ? L.aux_coef / ((float)L.Bfull * (float)L.aux_dim) : 0.f;
  const float (&t)[32] = smp.act;
  float la = 0.f, lx = 0.f, g[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) {
    const float e = o[j] - t[j];
    la += j < Aa ? e * e : 0.f;
    lx += (j >= Aa && j < A) ? e * e : 0.f;
    g[j] = j < Aa ? 2.f * sa * e : (j < A ? 2.f * sx * e : 0.f);
  }
#pragma unroll
  for (int j = 0; j < 32; j += 2) pk[j >> 1] = pack2bf(g[j], g[j + 1]);
  st[0] = la; st[1] = lx; st[2] = 0.f; st[3] = 0.f;
}

// Sums of the four statistics and (if dls_part) of the A log-std terms over the block, in a fixed
// order: xor-butterfly inside each wave (all sums side by side, so that their steps overlap), then
// the wave sums.  Every thread of the block calls this (threads without a sample pass zeros);
// wred: 4 x 36 floats of LDS.
__device__ __forceinline__ void loss_block_sums(const float (&st)[4], const float (&dls)[32], int A, float (*wred)[36],
                                                float* __restrict__ stat_part, float* __restrict__ dls_part) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  for (int i = tid; i < 4 * 36; i += blockDim.x) (&wred[0][0])[i] = 0.f;  // waves the block does not have contribute zero
  __syncthreads();
  float rv[36];
#pragma unroll
  for (int k = 0; k < 4; ++k) rv[k] = st[k];
#pragma unroll
  for (int j = 0; j < 32; ++j) rv[4 + j] = dls[j];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1)
#pragma unroll
    for (int k = 0; k < 36; ++k) rv[k] += __shfl_xor(rv[k], off);  // sums beyond 4 + A are zeros
  if (lane == 0 && wave < 4) {
#pragma unroll
    for (int k = 0; k < 36; ++k)
      if (k < 4 + A) wred[wave][k] = rv[k];
  }
  __syncthreads();
  if (tid < 4) stat_part[(int64_t)blockIdx.x * LOSS_NSTAT + tid] = (wred[0][tid] + wred[1][tid]) + (wred[2][tid] + wred[3][tid]);
  else if (dls_part && tid >= 32 && tid < 32 + A) {
    const int j = tid - 32;
    dls_part[(int64_t)blockIdx.x * 32 + j] = (wred[0][4 + j] + wred[1][4 + j]) + (wred[2][4 + j] + wred[3][4 + j]);
  }
}

// The losses on a chunk of `B` samples, one thread per sample (blocks of up to 256 threads): reads the
// head outputs out[b][0..32), writes the gradient rows dout[b][0..32) (bf16) and per-block partial
// sums of the statistics (and of dL/dlogstd for PPO).
template <bool DISTILL>
__global__ __launch_bounds__(256) void k_loss(int B, LossData L, const float* __restrict__ out, bf16_t* __restrict__ dout,
                                              float* __restrict__ stat_part, float* __restrict__ dls_part) {
  __shared__ float sig_inv[32], ls[32];
  __shared__ float wred[4][36];
  const int tid = threadIdx.x;
  if (!DISTILL && tid < L.A) { ls[tid] = L.logstd[tid]; sig_inv[tid] = __expf(-L.logstd[tid]); }
  __syncthreads();
  const int b = blockIdx.x * blockDim.x + tid;
  float st[4] = {0.f, 0.f, 0.f, 0.f}, dls[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) dls[j] = 0.f;
  if (b < B) {
    const int64_t s = L.idx[b];
    float o[HEAD_LD];  // the head's output row: eight 16-byte loads
#pragma unroll
    for (int q = 0; q < HEAD_LD / 4; ++q) {
      const float4 v4 = *reinterpret_cast<const float4*>(out + (int64_t)b * HEAD_LD + 4 * q);
      o[4 * q] = v4.x; o[4 * q + 1] = v4.y; o[4 * q + 2] = v4.z; o[4 * q + 3] = v4.w;
    }
    uint32_t pk[16];
    const LossSample smp = loss_gather(L, s, !DISTILL);
    if (DISTILL) mse_loss_sample(L, smp, o, pk, st);
    else ppo_loss_sample(L, sig_inv, ls, smp, o, pk, st, dls);
    // the row of 32 bf16 leaves as four 16-byte stores
    uint4* d = reinterpret_cast<uint4*>(dout + (int64_t)b * HEAD_LD);
#pragma unroll
    for (int q = 0; q < 4; ++q) d[q] = make_uint4(pk[4 * q], pk[4 * q + 1], pk[4 * q + 2], pk[4 * q + 3]);
  }
  loss_block_sums(st, dls, DISTILL ? 0 : L.A, wred, stat_part, DISTILL ? nullptr : dls_part);
}

// Device-side record of one optimiser step (mirrors the host ppo_mb_stats layout).
struct DevStats { float pi_loss, v_loss, entropy, approx_kl, clip_frac, grad_norm, total_loss; int32_t nonfinite; float lr; };

// Sum the per-block partials of one minibatch (all chunks) in block order; write the loss
// statistics and the log-std gradient (which also carries the entropy bonus).  The work of one
// block of 256 threads; it rides along as the last block of the backward pass's reduction launch.
// With desired_kl > 0 it also moves the learning rate kept in *lr_dev by the minibatch's approx_kl
// (above 2 desired_kl: / 1.5, not below lr_min; below desired_kl / 2: x 1.5, not above lr_max); the
// Adam step that follows reads the rate from there.  lr_reset: the rate starts from lr_init
// instead of the stored one (first step of an update).
struct LossFinalize {
  int on, nblocks, Bfull, A, distill;
  const float *stat_part, *dls_part, *logstd;
  float vf_coef, ent_coef;
  DevStats* st;
  float* g_logstd;
  float desired_kl, lr_min, lr_max, lr_init;
  int lr_reset;
  float* lr_dev;
  int aux_dim;     // distillation: auxiliary columns and their weight
  float aux_coef;
};
__device__ __forceinline__ void loss_finalize_block(const LossFinalize& f) {
  // column c (4 statistics, then the A log-std gradients) is summed by 8 lanes, lane j taking
  // blocks j, j+8, ... in order; the 8 sums are combined in a fixed order
  const int tid = threadIdx.x, l8 = tid & 7;
  __shared__ float tot[4];
  const int ncol = 4 + (f.distill ? 0 : f.A);
  for (int c0 = 0; c0 < ncol; c0 += 32) {
    const int col = c0 + (tid >> 3);
    float s = 0.f;
    if (col < ncol)
      for (int b = l8; b < f.nblocks; b += 8) s += col < 4 ? f.stat_part[(int64_t)b * LOSS_NSTAT + col] : f.dls_part[(int64_t)b * 32 + (col - 4)];
    s += __shfl_xor(s, 1); s += __shfl_xor(s, 2); s += __shfl_xor(s, 4);
    if (l8 == 0 && col < ncol) {
      if (col < 4) tot[col] = s;
      else f.g_logstd[col - 4] = s - f.ent_coef;
    }
  }
  __syncthreads();
  if (tid == 0) {
    DevStats* st = f.st;
    if (f.distill) {
      const float la = tot[0] / ((float)f.Bfull * (float)(f.A - f.aux_dim));
      const float lx = f.aux_dim > 0 ? tot[1] / ((float)f.Bfull * (float)f.aux_dim) : 0.f;
      st->pi_loss = la; st->v_loss = lx; st->entropy = 0.f; st->approx_kl = 0.f; st->clip_frac = 0.f;
      st->total_loss = f.aux_dim > 0 ? la + f.aux_coef * lx : la;
    } else {
      float invB = 1.f / (float)f.Bfull, ent = 0.f;
      for (int j = 0; j < f.A; ++j) ent += f.logstd[j] + 1.4189385332046727418f;
      st->pi_loss = tot[0] * invB; st->v_loss = tot[1] * invB; st->entropy = ent;
      st->approx_kl = tot[2] * invB; st->clip_frac = tot[3] * invB;
      st->total_loss = st->pi_loss + f.vf_coef * st->v_loss - f.ent_coef * ent;
    }
    float lr = f.lr_init;
    if (!f.distill && f.desired_kl > 0.f) {
      if (!f.lr_reset) lr = *f.lr_dev;
      const float kl = st->approx_kl;
      if (kl > 2.f * f.desired_kl) lr = fmaxf(f.lr_min, lr / 1.5f);
      else if (kl < 0.5f * f.desired_kl) lr = fminf(f.lr_max, lr * 1.5f);
      *f.lr_dev = lr;
    }
    st->lr = lr;
    st->nonfinite = isfinite(st->total_loss) ? 0 : 1;
  }
}

// ---------------------------------------------------------------- partial sums of a backward pass
// Every pending reduction of a backward pass in one launch: job j covers blocks [first[j], first[j+1]).
// kind 0: dst[i] (+)= sum_s partial[s][i]; kind 1: partials stored transposed, dst[n*K + k] (+)=
// sum_s partial[s][k*N + n]; kind 2: partial[s][co][K+1] of the first convolution, whose last column
// is the bias gradient (dst2).  Jobs with vec set (n a multiple of 4, partials 16-byte aligned) take
// four outputs per lane with 16-byte loads (128 outputs per block), the others one (32 per block).
struct ReduceJobs {
  static constexpr int MAXJ = 16;
  int njobs;
  int first[MAXJ + 1];
  int kind[MAXJ], splits[MAXJ], N[MAXJ], K[MAXJ], accumulate[MAXJ], vec[MAXJ];
  int64_t n[MAXJ];
  const float* partial[MAXJ];
  float* dst[MAXJ];
  float* dst2[MAXJ];
};
__global__ __launch_bounds__(256) void k_reduce_batch(ReduceJobs jobs, LossFinalize fin) {
  if (fin.on && blockIdx.x + 1 == gridDim.x) { loss_finalize_block(fin); return; }  // the block behind the last job
  __shared__ float red[8][33 * 4];
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first[j + 1]) ++j;
  const int64_t nn = jobs.n[j];
  const int kind = jobs.kind[j], blk = (int)blockIdx.x - jobs.first[j];
  auto put = [&](int64_t i, float s) {
    float* d;
    if (kind == 0) d = jobs.dst[j] + i;
    else if (kind == 1) { const int N = jobs.N[j], kk = (int)(i / N), n = (int)(i - (int64_t)kk * N); d = jobs.dst[j] + (int64_t)n * jobs.K[j] + kk; }
    else { const int KP = jobs.K[j] + 1, co = (int)(i / KP), k = (int)(i - (int64_t)co * KP); d = k == jobs.K[j] ? jobs.dst2[j] + co : jobs.dst[j] + (int64_t)co * jobs.K[j] + k; }
    *d = jobs.accumulate[j] ? *d + s : s;
  };
  if (jobs.vec[j]) {
    const int64_t i = ((int64_t)blk * 32 + (threadIdx.x & 31)) * 4;
    float s[4];
    reduce_partials_block<4>(jobs.partial[j], jobs.splits[j], nn, i, red, s);
    if (threadIdx.x < 32 && i < nn) {
#pragma unroll
      for (int w = 0; w < 4; ++w) put(i + w, s[w]);
    }
  } else {
    const int64_t i = (int64_t)blk * 32 + (threadIdx.x & 31);
    float s[1];
    reduce_partials_block<1>(jobs.partial[j], jobs.splits[j], nn, i, reinterpret_cast<float (*)[33]>(&red[0][0]), s);
    if (threadIdx.x < 32 && i < nn) put(i, s[0]);
  }
}


// ---------------------------------------------------------------- Adam
// m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; p -= lr (m/c1) / (sqrt(v/c2) + eps), c1 = 1-b1^k,
// c2 = 1-b2^k passed in.  Also refreshes the bf16 copy of the parameters and leaves per-block sums
// of g^2 for the gradient-norm statistic.  With gradient-norm clipping the gradient enters as
// g * *clip_coef (the coefficient min(1, c / (||g|| + 1e-6)) left by k_gnorm_finalize); the sums
// of g^2 are of the gradient before clipping either way.  lr_dev (if not null) holds the rate
// instead of the argument: the KL-adaptive schedule keeps it on the device.
__global__ __launch_bounds__(256) void k_adam(int64_t n, float* __restrict__ p, float* __restrict__ m,
                                              float* __restrict__ v, const float* __restrict__ g,
                                              bf16_t* __restrict__ shadow, float lr, float b1, float b2, float eps,
                                              float inv_c1, float inv_c2, float* __restrict__ sq_part,
                                              const float* __restrict__ clip_coef, const float* __restrict__ lr_dev) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  if (lr_dev) lr = *lr_dev;
  const float coef = clip_coef ? *clip_coef : 1.f;
  float sq = 0.f;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + tid) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    if (i + 4 <= n) {
      float4 g4 = *reinterpret_cast<const float4*>(g + i), m4 = *reinterpret_cast<float4*>(m + i);
      float4 v4 = *reinterpret_cast<float4*>(v + i), p4 = *reinterpret_cast<float4*>(p + i);
      float* gp = &g4.x; float* mp = &m4.x; float* vp = &v4.x; float* pp = &p4.x;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        sq += gp[j] * gp[j];
        const float gc = gp[j] * coef;
        mp[j] = b1 * mp[j] + (1.f - b1) * gc;
        vp[j] = b2 * vp[j] + (1.f - b2) * gc * gc;
        pp[j] -= lr * (mp[j] * inv_c1) / (sqrtf(vp[j] * inv_c2) + eps);
      }
      *reinterpret_cast<float4*>(m + i) = m4; *reinterpret_cast<float4*>(v + i) = v4; *reinterpret_cast<float4*>(p + i) = p4;
      uint2 s2; s2.x = pack2bf(p4.x, p4.y); s2.y = pack2bf(p4.z, p4.w);
      *reinterpret_cast<uint2*>(shadow + i) = s2;
    } else {
      for (int64_t q = i; q < n; ++q) {
        const float gr = g[q], gq = gr * coef;
        float mq = b1 * m[q] + (1.f - b1) * gq, vq = b2 * v[q] + (1.f - b2) * gq * gq;
        float pq = p[q] - lr * (mq * inv_c1) / (sqrtf(vq * inv_c2) + eps);
        m[q] = mq; v[q] = vq; p[q] = pq; shadow[q] = f2bf(pq); sq += gr * gr;
      }
    }
  }
  red[tid] = sq;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
  if (tid == 0) sq_part[blockIdx.x] = red[0];
}
// Per-block sums of g^2 with the blocking of k_adam (the same partial sums, so the norm used for
// clipping is bit-identical to the statistic reported without clipping).
__global__ __launch_bounds__(256) void k_gnorm_partial(int64_t n, const float* __restrict__ g, float* __restrict__ sq_part) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  float sq = 0.f;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + tid) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    if (i + 4 <= n) {
      const float4 g4 = *reinterpret_cast<const float4*>(g + i);
      sq += g4.x * g4.x; sq += g4.y * g4.y; sq += g4.z * g4.z; sq += g4.w * g4.w;
    } else {
      for (int64_t q = i; q < n; ++q) sq += g[q] * g[q];
    }
  }
  red[tid] = sq;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
  if (tid == 0) sq_part[blockIdx.x] = red[0];
}
// Gradient norm from the per-block sums; with max_norm > 0 also the clipping coefficient
// min(1, max_norm / (norm + 1e-6)) for k_adam.  The work of one block of 256 threads.
struct GnormFinalize { int on, nb; const float* sq_part; DevStats* st; float max_norm; float* clip_coef; };
__device__ __forceinline__ void gnorm_finalize_block(const GnormFinalize& f) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  float s = 0.f;
  for (int b = tid; b < f.nb; b += 256) s += f.sq_part[b];
  red[tid] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) { if (tid < w) red[tid] += red[tid + w]; __syncthreads(); }
  if (tid == 0) {
    const float norm = sqrtf(red[0]);
    f.st->grad_norm = norm;
    if (!isfinite(red[0])) f.st->nonfinite = 1;
    if (f.clip_coef) *f.clip_coef = f.max_norm > 0.f ? fminf(1.f, f.max_norm / (norm + 1e-6f)) : 1.f;
  }
}
__global__ __launch_bounds__(256) void k_gnorm_finalize(GnormFinalize f) { gnorm_finalize_block(f); }

// ---------------------------------------------------------------- advantage normalisation
// out = (adv - mean) / (std + 1e-8) over all S samples of the rollout, std the population standard deviation.
// Two launches of ADVN_BLOCKS-or-fewer blocks.  k_adv_stats: block b takes the contiguous slice b of the samples and
// leaves (count, mean, sum of squared deviations from its own mean) of it.  k_adv_apply: every block merges those
// triples in block order (the pairwise update of Chan et al. for combined means and variances: no cancellation
// between a large mean^2 and E[x^2]) and normalises its slice.  Fixed slices and a fixed merge order: the result
// does not depend on the launch.
#define ADVN_BLOCKS 256
__device__ __forceinline__ float block_sum_1024(float x, float* red) {
  const int tid = threadIdx.x;
  __syncthreads();
  red[tid] = x;
  __syncthreads();
  for (int w = 512; w > 0; w >>= 1) { if (tid < w) red[tid] += red[tid + w]; __syncthreads(); }
  return red[0];
}
__global__ __launch_bounds__(1024) void k_adv_stats(int S, int per, const float* __restrict__ adv, float* __restrict__ part) {
  __shared__ float red[1024];
  const int tid = threadIdx.x, b = blockIdx.x, lo = b * per, hi = lo + per < S ? lo + per : S, cnt = hi - lo;
  float s = 0.f;
  for (int i = lo + tid; i < hi; i += 1024) s += adv[i];
  const float mean = block_sum_1024(s, red) / (float)cnt;
  float q = 0.f;
  for (int i = lo + tid; i < hi; i += 1024) { const float d = adv[i] - mean; q += d * d; }
  const float m2 = block_sum_1024(q, red);
  if (tid == 0) { part[3 * b] = (float)cnt; part[3 * b + 1] = mean; part[3 * b + 2] = m2; }
}
__global__ __launch_bounds__(1024) void k_adv_apply(int S, int per, int nblk, const float* __restrict__ adv, const float* __restrict__ part,
                                                    float* __restrict__ out) {
  float n = part[0], mean = part[1], m2 = part[2];
  for (int b = 1; b < nblk; ++b) {
    const float nb = part[3 * b], mb = part[3 * b + 1], qb = part[3 * b + 2], nab = n + nb, dlt = mb - mean;
    mean += dlt * (nb / nab);
    m2 += qb + dlt * dlt * (n * nb / nab);
    n = nab;
  }
  const float inv = 1.f / (sqrtf(m2 / (float)S) + 1e-8f);
  const int lo = blockIdx.x * per, hi = lo + per < S ? lo + per : S;
  for (int i = lo + threadIdx.x; i < hi; i += 1024) out[i] = (adv[i] - mean) * inv;
}
__global__ void k_cast_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f2bf(src[i]);
}

// ---------------------------------------------------------------- weight re-packing for the backward GEMMs
// All per-update re-packs in one launch: job j covers blocks [first[j], first[j+1]).
// kind 0, transpose with zero padding (a = rows, b = cols, ld = leading dimension of dst):
//   dst[c][r] = src[r][c] for r < rows, zero for rows <= r < ld;
// kind 1, per-tap transpose for the quad-organised transposed convolution (a = Cout, b = Cin):
//   dst[(tap*Cin + ci)*Cout + co] = W[co][tap*Cin + ci].
struct RepackJobs {
  static constexpr int MAXJ = 12;
  int njobs;
  int first[MAXJ + 1];
  int kind[MAXJ], a[MAXJ], b[MAXJ], ld[MAXJ];
  const bf16_t* src[MAXJ];
  bf16_t* dst[MAXJ];
};
__global__ __launch_bounds__(256) void k_repack_all(RepackJobs jobs, GnormFinalize gn) {
  if (gn.on && blockIdx.x + 1 == gridDim.x) { gnorm_finalize_block(gn); return; }  // the block behind the last job: the step's gradient norm
  int j = 0;
  while (j + 1 < jobs.njobs && (int)blockIdx.x >= jobs.first[j + 1]) ++j;
  const int64_t i = (int64_t)((int)blockIdx.x - jobs.first[j]) * 256 + threadIdx.x;
  const bf16_t* __restrict__ src = jobs.src[j];
  bf16_t* __restrict__ dst = jobs.dst[j];
  if (jobs.kind[j] == 0) {
    const int rows = jobs.a[j], cols = jobs.b[j], ld_dst = jobs.ld[j];
    if (i >= (int64_t)cols * ld_dst) return;
    const int c = (int)(i / ld_dst), r = (int)(i - (int64_t)c * ld_dst);
    dst[i] = r < rows ? src[(int64_t)r * cols + c] : (bf16_t)0;
  } else {
    const int Cout = jobs.a[j], Cin = jobs.b[j];
    if (i >= (int64_t)9 * Cin * Cout) return;
    const int tap = (int)(i / ((int64_t)Cin * Cout)), rem = (int)(i - (int64_t)tap * Cin * Cout), ci = rem / Cout, co = rem - ci * Cout;
    dst[i] = src[(int64_t)co * 9 * Cin + tap * Cin + ci];
  }
}

// dst[px*Cin + ci][(tu*2 + dx)*Cout + co] = W[co][(u*3+v)*Cin + ci] with u = py ? 2*tu : 1 and the
// column tap v given by (px, dx): even pixel (px = 0) takes v = 1 from dx = 0 and nothing from
// dx = 1; odd pixel takes v = 2 from dx = 0 and v = 0 from dx = 1.
__global__ void k_pack_dgrad_w(const bf16_t* __restrict__ w, int Cout, int Cin, int py, bf16_t* __restrict__ dst) {
  const int Kc = (1 + py) * 2 * Cout;
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)2 * Cin * Kc) return;
  int n = (int)(i / Kc), k = (int)(i - (int64_t)n * Kc), px = n / Cin, ci = n - px * Cin;
  int t = k / Cout, co = k - t * Cout, tu = t >> 1, dx = t & 1;
  int u = py ? 2 * tu : 1;
  int v = px ? (dx ? 0 : 2) : (dx ? -1 : 1);
  dst[i] = v < 0 ? (bf16_t)0 : w[(int64_t)co * 9 * Cin + (u * 3 + v) * Cin + ci];
}
