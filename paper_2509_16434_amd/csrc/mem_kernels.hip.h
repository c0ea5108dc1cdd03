// Bandwidth-bound and elementwise kernels of the learner: buffer append, GAE scan, minibatch
// permutation, first-layer convolution (K = 9 or 27: too thin for MFMA), losses, Adam and
// weight re-packing.
#pragma once
#include "common.hip.h"

// ---------------------------------------------------------------- buffer append
// One step's images [N][V][C][HW] (fp32 or bf16) -> bf16 channel-last [N][V][HW][C] at the
// step's slab.  Each thread converts 8 consecutive pixels of one (n, v) image.
template <typename InT>
__global__ void k_write_obs(const InT* __restrict__ src, bf16_t* __restrict__ dst, int64_t n_img, int C, int HW) {
  const int groups = (HW + 7) / 8;
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

// Per-step scalars: proprio -> bf16, action/logp/value/reward fp32, done u8.
__global__ void k_write_scalars(int N, int P, int A, const float* __restrict__ proprio, const float* __restrict__ action,
                                const float* __restrict__ logp, const float* __restrict__ value,
                                const float* __restrict__ reward, const uint8_t* __restrict__ done,
                                bf16_t* __restrict__ o_proprio, float* __restrict__ o_action, float* __restrict__ o_logp,
                                float* __restrict__ o_value, float* __restrict__ o_reward, uint8_t* __restrict__ o_done) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < (int64_t)N * P) o_proprio[i] = f2bf(proprio[i]);
  if (i < (int64_t)N * A) o_action[i] = action[i];
  if (i < N) {
    if (logp) o_logp[i] = logp[i];
    if (value) o_value[i] = value[i];
    if (reward) o_reward[i] = reward[i];
    if (done) o_done[i] = done[i];
  }
}

// ---------------------------------------------------------------- GAE
// One thread per environment, reverse scan over time held in registers; at every t the
// wave reads/writes N-contiguous rows.
__global__ void k_gae(int T, int N, const float* __restrict__ reward, const uint8_t* __restrict__ done,
                      const float* __restrict__ value, const float* __restrict__ last_value, float gamma, float lambda,
                      float* __restrict__ adv, float* __restrict__ ret) {
  int n = blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= N) return;
  float next_v = last_value[n], next_a = 0.f;
  for (int t = T - 1; t >= 0; --t) {
    int64_t i = (int64_t)t * N + n;
    float nt = done[i] ? 0.f : 1.f, v = value[i];
    float delta = reward[i] + gamma * next_v * nt - v;
    float a = delta + gamma * lambda * nt * next_a;
    adv[i] = a; ret[i] = a + v;
    next_a = a; next_v = v;
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
__global__ void k_iota_i32(int32_t* p, int n, int32_t first) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = first + i;
}
__global__ void k_perm_hist(uint64_t stream, int S, int shift, int32_t* __restrict__ hist) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S) return;
  int b = shift >= 64 ? 0 : (int)(perm_key(stream, (uint64_t)i) >> shift);
  atomicAdd(&hist[b], 1);
}
// exclusive scan of hist[nb] into start[nb]; one block of 1024 threads
__global__ void k_perm_scan(const int32_t* __restrict__ hist, int32_t* __restrict__ start, int nb) {
  __shared__ int32_t part[1024];
  int tid = threadIdx.x, per = (nb + 1023) / 1024, b0 = tid * per, s = 0;
  for (int j = 0; j < per; ++j) if (b0 + j < nb) s += hist[b0 + j];
  part[tid] = s;
  __syncthreads();
  if (tid == 0) { int run = 0; for (int j = 0; j < 1024; ++j) { int v = part[j]; part[j] = run; run += v; } }
  __syncthreads();
  int run = part[tid];
  for (int j = 0; j < per; ++j) if (b0 + j < nb) { start[b0 + j] = run; run += hist[b0 + j]; }
}
__global__ void k_perm_scatter(uint64_t stream, int S, int shift, const int32_t* __restrict__ start,
                               int32_t* __restrict__ cursor, int32_t* __restrict__ tmp) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= S) return;
  int b = shift >= 64 ? 0 : (int)(perm_key(stream, (uint64_t)i) >> shift);
  int pos = start[b] + atomicAdd(&cursor[b], 1);
  tmp[pos] = i;
}
__global__ void k_perm_rank(uint64_t stream, int S, int shift, const int32_t* __restrict__ start,
                            const int32_t* __restrict__ hist, const int32_t* __restrict__ tmp, int32_t* __restrict__ perm) {
  int p = blockIdx.x * blockDim.x + threadIdx.x;
  if (p >= S) return;
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
// 3x3 stride-2 pad-1 convolution of a 1- or 3-channel image read straight from the rollout
// buffer through the minibatch index (the gather is fused into the loader).  One thread per
// output pixel computes all Cout channels in fp32 and stores them channel-last as bf16.
// Weights are the fp32 master copy in [Cout][9*Cin] order, staged in LDS as [k][Cout].
template <int CIN>
__global__ __launch_bounds__(256) void k_conv1_fwd(ImgAddr in, int n_img, int H, int W, int Ho, int Wo, int Cout,
                                                   const float* __restrict__ Wt, const float* __restrict__ bias,
                                                   bf16_t* __restrict__ out) {
  constexpr int K = 9 * CIN;
  extern __shared__ float smem[];  // [K][Cout] weights, then [Cout] bias
  float* w = smem; float* bs = smem + K * Cout;
  for (int i = threadIdx.x; i < K * Cout; i += blockDim.x) { int co = i / K, k = i - co * K; w[k * Cout + co] = Wt[i]; }
  for (int i = threadIdx.x; i < Cout; i += blockDim.x) bs[i] = bias[i];
  __syncthreads();
  int64_t m = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  int64_t M = (int64_t)n_img * Ho * Wo;
  if (m >= M) return;
  int hw = Ho * Wo, img = (int)(m / hw), q = (int)(m - (int64_t)img * hw), oy = q / Wo, ox = q - oy * Wo;
  const bf16_t* p = in.ptr(img);
  float x[K];
#pragma unroll
  for (int u = 0; u < 3; ++u)
#pragma unroll
    for (int v = 0; v < 3; ++v) {
      int iy = 2 * oy - 1 + u, ix = 2 * ox - 1 + v;
      bool ok = (unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W;
#pragma unroll
      for (int c = 0; c < CIN; ++c) x[(u * 3 + v) * CIN + c] = ok ? bf2f(p[((int64_t)iy * W + ix) * CIN + c]) : 0.f;
    }
  bf16_t* o = out + m * Cout;
  for (int c0 = 0; c0 < Cout; c0 += 8) {
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = bs[c0 + j];
#pragma unroll
    for (int k = 0; k < K; ++k)
#pragma unroll
      for (int j = 0; j < 8; ++j) acc[j] += x[k] * w[k * Cout + c0 + j];
    uint4 pk;
    pk.x = pack2bf(fmaxf(acc[0], 0.f), fmaxf(acc[1], 0.f)); pk.y = pack2bf(fmaxf(acc[2], 0.f), fmaxf(acc[3], 0.f));
    pk.z = pack2bf(fmaxf(acc[4], 0.f), fmaxf(acc[5], 0.f)); pk.w = pack2bf(fmaxf(acc[6], 0.f), fmaxf(acc[7], 0.f));
    *reinterpret_cast<uint4*>(o + c0) = pk;
  }
}

// Weight/bias gradient of the first convolution: dW[co][k] = sum_m dY[m][co] * x[m][k], db[co] =
// sum_m dY[m][co].  TPP = Cout/COG threads share a pixel, each owning COG output channels and all
// 9*CIN taps (+1 bias column) as a register tile; a block walks its pixel range, then the tiles
// are summed across the wave with xor-shuffles, across the four waves through LDS, and written as
// one partial per block (summed later in block order).
template <int CIN, int COG>
__global__ __launch_bounds__(256) void k_conv1_wgrad(ImgAddr in, int n_img, int H, int W, int Ho, int Wo, int Cout,
                                                     const bf16_t* __restrict__ dy, int pixels_per_block,
                                                     float* __restrict__ partial) {
  constexpr int K = 9 * CIN, KP = K + 1;
  __shared__ float wsum[4 * 64 * KP];
  const int TPP = Cout / COG, PPI = 256 / TPP;
  const int tid = threadIdx.x, cg = tid % TPP, pl = tid / TPP;
  float acc[COG][KP];
#pragma unroll
  for (int j = 0; j < COG; ++j)
#pragma unroll
    for (int k = 0; k < KP; ++k) acc[j][k] = 0.f;
  const int64_t M = (int64_t)n_img * Ho * Wo;
  const int64_t mbeg = (int64_t)blockIdx.x * pixels_per_block;
  const int64_t mend = (mbeg + pixels_per_block < M) ? mbeg + pixels_per_block : M;
  int64_t m = mbeg + pl;
  const int hw = Ho * Wo;
  int img = (int)(m / hw), q = (int)(m - (int64_t)img * hw), oy = q / Wo, ox = q - oy * Wo;
  const bf16_t* p = (m < mend) ? in.ptr(img) : nullptr;
  for (; m < mend; m += PPI) {
    float x[K];
#pragma unroll
    for (int u = 0; u < 3; ++u)
#pragma unroll
      for (int v = 0; v < 3; ++v) {
        const int iy = 2 * oy - 1 + u, ix = 2 * ox - 1 + v;
        const bool ok = (unsigned)iy < (unsigned)H && (unsigned)ix < (unsigned)W;
#pragma unroll
        for (int c = 0; c < CIN; ++c) x[(u * 3 + v) * CIN + c] = ok ? bf2f(p[((int64_t)iy * W + ix) * CIN + c]) : 0.f;
      }
    float d[COG];
    const bf16_t* dp = dy + m * Cout + cg * COG;
    if constexpr (COG == 8) {
      uint4 r = *reinterpret_cast<const uint4*>(dp);
      const uint32_t w4[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) { d[2 * j] = __uint_as_float(w4[j] << 16); d[2 * j + 1] = __uint_as_float(w4[j] & 0xffff0000u); }
    } else {
      uint2 r = *reinterpret_cast<const uint2*>(dp);
      d[0] = __uint_as_float(r.x << 16); d[1] = __uint_as_float(r.x & 0xffff0000u);
      d[2] = __uint_as_float(r.y << 16); d[3] = __uint_as_float(r.y & 0xffff0000u);
    }
#pragma unroll
    for (int j = 0; j < COG; ++j) {
#pragma unroll
      for (int k = 0; k < K; ++k) acc[j][k] += d[j] * x[k];
      acc[j][K] += d[j];
    }
    // next pixel of this thread
    ox += PPI;
    while (ox >= Wo) { ox -= Wo; ++oy; }
    if (oy >= Ho) {
      while (oy >= Ho) { oy -= Ho; ++img; }
      p = (m + PPI < mend) ? in.ptr(img) : nullptr;
    }
  }
  // sum over the lanes of the wave that share cg (lane = (pl % (64/TPP)) * TPP + cg)
#pragma unroll
  for (int j = 0; j < COG; ++j)
#pragma unroll
    for (int k = 0; k < KP; ++k) {
      float v = acc[j][k];
      for (int off = TPP; off < 64; off <<= 1) v += __shfl_xor(v, off);
      acc[j][k] = v;
    }
  const int lane = tid & 63, wave = tid >> 6, npair = Cout * KP;
  if (lane < TPP) {
#pragma unroll
    for (int j = 0; j < COG; ++j)
#pragma unroll
      for (int k = 0; k < KP; ++k) wsum[wave * npair + (cg * COG + j) * KP + k] = acc[j][k];
  }
  __syncthreads();
  float* P = partial + (int64_t)blockIdx.x * npair;
  for (int pr = tid; pr < npair; pr += 256) P[pr] = (wsum[pr] + wsum[npair + pr]) + (wsum[2 * npair + pr] + wsum[3 * npair + pr]);
}
// Sum conv1 partials: partial[nb][Cout][K+1] -> gw[Cout][K], gb[Cout].  One block per output
// element; strided partial sums, then a fixed-order tree.
__global__ __launch_bounds__(256) void k_conv1_wgrad_reduce(const float* __restrict__ partial, int nb, int Cout, int K,
                                                            float* __restrict__ gw, float* __restrict__ gb, int accumulate) {
  __shared__ float red[256];
  const int pr = blockIdx.x, KP = K + 1, npair = Cout * KP, tid = threadIdx.x;
  float s = 0.f;
  for (int b = tid; b < nb; b += 256) s += partial[(int64_t)b * npair + pr];
  red[tid] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) { if (tid < w) red[tid] += red[tid + w]; __syncthreads(); }
  if (tid == 0) {
    const int co = pr / KP, k = pr - co * KP;
    float* dst = (k == K) ? gb + co : gw + co * K + k;
    *dst = (accumulate ? *dst : 0.f) + red[0];
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

// ---------------------------------------------------------------- losses
#define LOSS_NSTAT 8  // pi, v, kl, clipfrac sums; slots 4..7 unused
#define HEAD_LD 32    // row stride of the head output / head gradient matrices

// Clipped-surrogate PPO loss on a chunk of `B` samples of a minibatch of `Bfull`:
//   logp = sum_j [-z_j^2/2 - logstd_j - ln(2 pi)/2], z = (a - mu)/sigma; rho = exp(logp - logp_old)
//   L_pi = -mean min(rho A, clip(rho, 1-eps, 1+eps) A);  L_V = mean (V-R)^2 or its clipped max form
// One thread per sample.  Writes the gradient rows dOut[b][0..A) = dL/dmu, dOut[b][A] = dL/dV (bf16,
// zero padded to 32 columns) and per-block partial sums of the statistics and of dL/dlogstd.
__global__ __launch_bounds__(256) void k_ppo_loss(int B, int Bfull, int A, const float* __restrict__ out,
                                                  const float* __restrict__ logstd, const int32_t* __restrict__ idx,
                                                  const float* __restrict__ action, const float* __restrict__ logp_old,
                                                  const float* __restrict__ v_old, const float* __restrict__ adv,
                                                  const float* __restrict__ ret, float clip_eps, float vclip_eps,
                                                  float vf_coef, bf16_t* __restrict__ dout, float* __restrict__ stat_part,
                                                  float* __restrict__ dls_part) {
  __shared__ float red[256];
  __shared__ float sig_inv[32], ls[32];
  const int tid = threadIdx.x;
  if (tid < A) { ls[tid] = logstd[tid]; sig_inv[tid] = __expf(-logstd[tid]); }
  __syncthreads();
  const int b = blockIdx.x * 256 + tid;
  const bool ok = b < B;
  float st[4] = {0.f, 0.f, 0.f, 0.f};
  float dlogp = 0.f;
  float z[32];
  const float invB = 1.f / (float)Bfull;
  if (ok) {
    const int64_t s = idx[b];
    const float* o = out + (int64_t)b * HEAD_LD;
    float logp = 0.f;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      if (j < A) {
        z[j] = (action[s * A + j] - o[j]) * sig_inv[j];
        logp += -0.5f * z[j] * z[j] - ls[j] - 0.91893853320467274178f;
      } else z[j] = 0.f;
    }
    const float lr = logp - logp_old[s], rho = expf(lr), a = adv[s];
    const float rc = fminf(fmaxf(rho, 1.f - clip_eps), 1.f + clip_eps);
    const float s1 = rho * a, s2 = rc * a;
    st[0] = -fminf(s1, s2);
    dlogp = (s1 <= s2) ? -invB * a * rho : 0.f;
    st[2] = (rho - 1.f) - lr;
    st[3] = fabsf(rho - 1.f) > clip_eps ? 1.f : 0.f;
    const float v = o[A], r = ret[s], err = v - r;
    float dv;
    if (vclip_eps > 0.f) {
      const float d = v - v_old[s], dc = fminf(fmaxf(d, -vclip_eps), vclip_eps), errc = v_old[s] + dc - r;
      if (errc * errc > err * err) { st[1] = errc * errc; dv = (d >= -vclip_eps && d <= vclip_eps) ? 2.f * errc : 0.f; }
      else { st[1] = err * err; dv = 2.f * err; }
    } else { st[1] = err * err; dv = 2.f * err; }
    bf16_t* d = dout + (int64_t)b * HEAD_LD;
#pragma unroll
    for (int j = 0; j < 32; ++j) {
      float g = 0.f;
      if (j < A) g = dlogp * z[j] * sig_inv[j];
      else if (j == A) g = vf_coef * invB * dv;
      d[j] = f2bf(g);
    }
  }
  // block reductions in a fixed tree order
  auto block_sum = [&](float v) -> float {
    red[tid] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
    float r = red[0];
    __syncthreads();
    return r;
  };
  for (int k = 0; k < 4; ++k) { float r = block_sum(st[k]); if (tid == 0) stat_part[(int64_t)blockIdx.x * LOSS_NSTAT + k] = r; }
  for (int j = 0; j < A; ++j) {
    float r = block_sum(ok ? dlogp * (z[j] * z[j] - 1.f) : 0.f);
    if (tid == 0) dls_part[(int64_t)blockIdx.x * 32 + j] = r;
  }
}

// Distillation loss: mean over batch and action dims of (pred - teacher)^2.
__global__ __launch_bounds__(256) void k_mse_loss(int B, int Bfull, int A, const float* __restrict__ out,
                                                  const int32_t* __restrict__ idx, const float* __restrict__ teacher,
                                                  bf16_t* __restrict__ dout, float* __restrict__ stat_part) {
  __shared__ float red[256];
  const int tid = threadIdx.x, b = blockIdx.x * 256 + tid;
  float l = 0.f;
  const float sc = 1.f / ((float)Bfull * (float)A);
  if (b < B) {
    const int64_t s = idx[b];
    const float* o = out + (int64_t)b * HEAD_LD;
    bf16_t* d = dout + (int64_t)b * HEAD_LD;
    for (int j = 0; j < 32; ++j) {
      float g = 0.f;
      if (j < A) { float e = o[j] - teacher[s * A + j]; l += e * e; g = 2.f * sc * e; }
      d[j] = f2bf(g);
    }
  }
  red[tid] = l;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
  if (tid == 0) {
    float* sp = stat_part + (int64_t)blockIdx.x * LOSS_NSTAT;
    sp[0] = red[0]; sp[1] = 0.f; sp[2] = 0.f; sp[3] = 0.f;
  }
}

// Device-side record of one optimiser step (mirrors the host ppo_mb_stats layout).
struct DevStats { float pi_loss, v_loss, entropy, approx_kl, clip_frac, grad_norm, total_loss; int32_t nonfinite; };

// Sum the per-block partials of one minibatch (all chunks) in block order; write the loss
// statistics and the log-std gradient (which also carries the entropy bonus).
__global__ void k_loss_finalize(int nblocks, int Bfull, int A, int distill, const float* __restrict__ stat_part,
                                const float* __restrict__ dls_part, const float* __restrict__ logstd, float vf_coef,
                                float ent_coef, DevStats* __restrict__ st, float* __restrict__ g_logstd) {
  const int tid = threadIdx.x;
  __shared__ float tot[4];
  if (tid < 4) {
    float s = 0.f;
    for (int b = 0; b < nblocks; ++b) s += stat_part[(int64_t)b * LOSS_NSTAT + tid];
    tot[tid] = s;
  } else if (!distill && tid >= 32 && tid < 32 + A) {
    int j = tid - 32;
    float s = 0.f;
    for (int b = 0; b < nblocks; ++b) s += dls_part[(int64_t)b * 32 + j];
    g_logstd[j] = s - ent_coef;
  }
  __syncthreads();
  if (tid == 0) {
    if (distill) {
      float l = tot[0] / ((float)Bfull * (float)A);
      st->pi_loss = l; st->v_loss = 0.f; st->entropy = 0.f; st->approx_kl = 0.f; st->clip_frac = 0.f; st->total_loss = l;
    } else {
      float invB = 1.f / (float)Bfull, ent = 0.f;
      for (int j = 0; j < A; ++j) ent += logstd[j] + 1.4189385332046727418f;
      st->pi_loss = tot[0] * invB; st->v_loss = tot[1] * invB; st->entropy = ent;
      st->approx_kl = tot[2] * invB; st->clip_frac = tot[3] * invB;
      st->total_loss = st->pi_loss + vf_coef * st->v_loss - ent_coef * ent;
    }
    st->nonfinite = isfinite(st->total_loss) ? 0 : 1;
  }
}

// ---------------------------------------------------------------- Adam
// m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2; p -= lr (m/c1) / (sqrt(v/c2) + eps), c1 = 1-b1^k,
// c2 = 1-b2^k passed in.  Also refreshes the bf16 copy of the parameters and leaves per-block sums
// of g^2 for the gradient-norm statistic.
__global__ __launch_bounds__(256) void k_adam(int64_t n, float* __restrict__ p, float* __restrict__ m,
                                              float* __restrict__ v, const float* __restrict__ g,
                                              bf16_t* __restrict__ shadow, float lr, float b1, float b2, float eps,
                                              float inv_c1, float inv_c2, float* __restrict__ sq_part) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  float sq = 0.f;
  for (int64_t i = ((int64_t)blockIdx.x * 256 + tid) * 4; i < n; i += (int64_t)gridDim.x * 1024) {
    if (i + 4 <= n) {
      float4 g4 = *reinterpret_cast<const float4*>(g + i), m4 = *reinterpret_cast<float4*>(m + i);
      float4 v4 = *reinterpret_cast<float4*>(v + i), p4 = *reinterpret_cast<float4*>(p + i);
      float* gp = &g4.x; float* mp = &m4.x; float* vp = &v4.x; float* pp = &p4.x;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        mp[j] = b1 * mp[j] + (1.f - b1) * gp[j];
        vp[j] = b2 * vp[j] + (1.f - b2) * gp[j] * gp[j];
        pp[j] -= lr * (mp[j] * inv_c1) / (sqrtf(vp[j] * inv_c2) + eps);
        sq += gp[j] * gp[j];
      }
      *reinterpret_cast<float4*>(m + i) = m4; *reinterpret_cast<float4*>(v + i) = v4; *reinterpret_cast<float4*>(p + i) = p4;
      uint2 s2; s2.x = pack2bf(p4.x, p4.y); s2.y = pack2bf(p4.z, p4.w);
      *reinterpret_cast<uint2*>(shadow + i) = s2;
    } else {
      for (int64_t q = i; q < n; ++q) {
        float gq = g[q];
        float mq = b1 * m[q] + (1.f - b1) * gq, vq = b2 * v[q] + (1.f - b2) * gq * gq;
        float pq = p[q] - lr * (mq * inv_c1) / (sqrtf(vq * inv_c2) + eps);
        m[q] = mq; v[q] = vq; p[q] = pq; shadow[q] = f2bf(pq); sq += gq * gq;
      }
    }
  }
  red[tid] = sq;
  __syncthreads();
  for (int s = 128; s > 0; s >>= 1) { if (tid < s) red[tid] += red[tid + s]; __syncthreads(); }
  if (tid == 0) sq_part[blockIdx.x] = red[0];
}
__global__ __launch_bounds__(256) void k_gnorm_finalize(const float* __restrict__ sq_part, int nb, DevStats* __restrict__ st) {
  __shared__ float red[256];
  const int tid = threadIdx.x;
  float s = 0.f;
  for (int b = tid; b < nb; b += 256) s += sq_part[b];
  red[tid] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) { if (tid < w) red[tid] += red[tid + w]; __syncthreads(); }
  if (tid == 0) {
    st->grad_norm = sqrtf(red[0]);
    if (!isfinite(red[0])) st->nonfinite = 1;
  }
}
__global__ void k_cast_bf16(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = f2bf(src[i]);
}

// ---------------------------------------------------------------- weight re-packing for the backward GEMMs
// dst[c][r] = src[r][c] for r < rows, zero for rows <= r < ld_dst.
__global__ void k_transpose_bf16(const bf16_t* __restrict__ src, int rows, int cols, bf16_t* __restrict__ dst, int ld_dst) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)cols * ld_dst) return;
  int c = (int)(i / ld_dst), r = (int)(i - (int64_t)c * ld_dst);
  dst[i] = r < rows ? src[(int64_t)r * cols + c] : (bf16_t)0;
}
// Transposed-convolution weights of row parity py for pixel-pair rows:
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
