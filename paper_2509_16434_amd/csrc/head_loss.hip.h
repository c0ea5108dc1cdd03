// The network's output layer (policy means and value: NH <= 32 columns), the loss, and the output
// layer's backward in one kernel.  Each of these is tiny; as separate launches (a GEMM, the loss, a
// weight-gradient GEMM with its partial sums, an input-gradient GEMM) their fixed costs dominate an
// optimiser step at small batch sizes.
//
// A block of 256 threads takes 64 samples:
//   1. the samples' last hidden activations H (64 x HID bf16) and the head weights W (NH x HID) go to LDS;
//   2. O = H W^T + b (fp32) with 32x32x16 MFMAs (waves 0 and 1, 32 samples each);
//   3. wave 0, one lane per sample, evaluates the loss: the gradient row dO (bf16, 32 columns) stays in
//      LDS, the loss statistics leave as one partial per block;
//   4. dH = dO W, masked by H > 0 (ReLU), rounded to bf16, staged and written out as full rows
//      (wave w: hidden units 32w .. 32w+31);
//   5. this block's term of dW = dO^T H (contraction over the 64 samples; both operands are row-major
//      over samples and are read with transposing LDS reads, as in k_wgrad) and of db = column sums
//      of dO leave as fp32 partials, summed afterwards in block order.
// Operand rounding is that of the separate kernels: bf16 H, W, dO and dH, fp32 accumulation.
#pragma once
#include "gemm.hip.h"
#include "mem_kernels.hip.h"

struct HeadLossArgs {
  const bf16_t* h;        // [n][HID] last hidden activations (after ReLU)
  const bf16_t* w;        // [NH][HID] head weights
  const bf16_t* wt;       // [HID][32] their transpose, zero padded
  const float* bias;      // [NH]
  bf16_t* dh;             // [n][HID] gradient of h, ReLU-masked
  float* wpart;           // [gridDim.x][NH][HID]
  float* bpart;           // [gridDim.x][NH]
  float* stat_part;       // [gridDim.x][LOSS_NSTAT]
  float* dls_part;        // [gridDim.x][32] (PPO only)
  int n, NH;
};

template <int HID>
struct HeadLossShape {
  static constexpr int HPA = HID + 8;    // pitch of the copy read row-wise (16 bytes mod 256: 16 rows tile the banks)
  static constexpr int HPB = HID + 32;   // pitch of the copy read through transposing reads (64 bytes mod 256)
  static constexpr int DPA = 40, DPB = 96;
  static constexpr int OFF_HA = 0, OFF_HB = OFF_HA + 64 * HPA * 2, OFF_W = OFF_HB + 64 * HPB * 2, OFF_O = OFF_W + 32 * HPA * 2;
  static constexpr int OFF_DA = OFF_O + 64 * 33 * 4, OFF_DB = OFF_DA + 64 * DPA * 2, OFF_DH = OFF_DB + 64 * DPB * 2, OFF_RED = OFF_DH + 64 * HPA * 2;
  static constexpr int LDS_BYTES = OFF_RED + (4 * 36 + 64) * 4;
};

template <int HID, bool DISTILL>
__global__ __launch_bounds__(256) void k_head_loss(HeadLossArgs a, LossData L) {
  typedef HeadLossShape<HID> S;
  static_assert(HID % 32 == 0 && HID >= 32 && HID <= 128, "one 32-wide tile of hidden units per wave");
  constexpr int HPA = S::HPA, HPB = S::HPB, DPA = S::DPA, DPB = S::DPB, NT = HID / 32;
  extern __shared__ __attribute__((aligned(16))) char lds[];
  bf16_t* const Ha = reinterpret_cast<bf16_t*>(lds + S::OFF_HA);
  bf16_t* const Hb = reinterpret_cast<bf16_t*>(lds + S::OFF_HB);
  bf16_t* const Ws = reinterpret_cast<bf16_t*>(lds + S::OFF_W);
  float* const Os = reinterpret_cast<float*>(lds + S::OFF_O);
  bf16_t* const Da = reinterpret_cast<bf16_t*>(lds + S::OFF_DA);
  bf16_t* const Db = reinterpret_cast<bf16_t*>(lds + S::OFF_DB);
  bf16_t* const DHs = reinterpret_cast<bf16_t*>(lds + S::OFF_DH);
  float (*wred)[36] = reinterpret_cast<float (*)[36]>(lds + S::OFF_RED);
  float* const sgl = reinterpret_cast<float*>(lds + S::OFF_RED) + 4 * 36;  // sig_inv[32], ls[32]
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, h = lane >> 5;
  const int s0 = blockIdx.x * 64, ns = min(64, a.n - s0);  // this block's samples

  // the loss's gathers from the rollout start now: their latency passes during steps 1 and 2
  LossSample smp;
  if (wave == 0 && lane < ns) smp = loss_gather(L, (int64_t)L.idx[s0 + lane], !DISTILL);

  // ---- 1. H rows (zeros beyond the chunk) in both pitches, W rows (zeros beyond NH)
  constexpr int CPR = HID / 8;  // 16-byte chunks per row
  for (int c = tid; c < 64 * CPR; c += 256) {
    const int r = c / CPR, cg = c - r * CPR;
    const uint4 v = r < ns ? *reinterpret_cast<const uint4*>(a.h + (int64_t)(s0 + r) * HID + cg * 8) : make_uint4(0u, 0u, 0u, 0u);
    *reinterpret_cast<uint4*>(Ha + r * HPA + cg * 8) = v;
    *reinterpret_cast<uint4*>(Hb + r * HPB + cg * 8) = v;
  }
  for (int c = tid; c < 32 * CPR; c += 256) {
    const int r = c / CPR, cg = c - r * CPR;
    *reinterpret_cast<uint4*>(Ws + r * HPA + cg * 8) = r < a.NH ? *reinterpret_cast<const uint4*>(a.w + (int64_t)r * HID + cg * 8) : make_uint4(0u, 0u, 0u, 0u);
  }
  if (!DISTILL && tid < L.A) { sgl[32 + tid] = L.logstd[tid]; sgl[tid] = __expf(-L.logstd[tid]); }
  __syncthreads();

  // ---- 2. O[s][j] = sum_k H[s][k] W[j][k] + b[j]: wave t < 2 takes samples 32t .. 32t+31
  if (wave < 2) {
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < HID / 16; ++ks) {
      const bf16x8_t bw = *reinterpret_cast<const bf16x8_t*>(Ws + l32 * HPA + ks * 16 + h * 8);
      const bf16x8_t ah = *reinterpret_cast<const bf16x8_t*>(Ha + (wave * 32 + l32) * HPA + ks * 16 + h * 8);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bw, ah, acc, 0, 0, 0);
    }
    // acc[g*4+q] = O[sample wave*32 + l32][column g*8 + h*4 + q]
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int j = (e >> 2) * 8 + h * 4 + (e & 3);
      Os[(wave * 32 + l32) * 33 + j] = acc[e] + (j < a.NH ? a.bias[j] : 0.f);
    }
  }
  __syncthreads();

  // ---- 3. the loss, one lane of wave 0 per sample
  float st[4] = {0.f, 0.f, 0.f, 0.f}, dls[32];
#pragma unroll
  for (int j = 0; j < 32; ++j) dls[j] = 0.f;
  if (wave == 0) {
    uint32_t pk[16];
#pragma unroll
    for (int q = 0; q < 16; ++q) pk[q] = 0u;
    if (lane < ns) {
      float o[HEAD_LD];
#pragma unroll
      for (int j = 0; j < HEAD_LD; ++j) o[j] = Os[lane * 33 + j];
      if (DISTILL) mse_loss_sample(L, smp, o, pk, st);
      else ppo_loss_sample(L, sgl, sgl + 32, smp, o, pk, st, dls);
    }
    // the gradient row (zeros for lanes beyond the chunk) in both pitches
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const uint4 v = make_uint4(pk[4 * q], pk[4 * q + 1], pk[4 * q + 2], pk[4 * q + 3]);
      *reinterpret_cast<uint4*>(Da + lane * DPA + q * 8) = v;
      *reinterpret_cast<uint4*>(Db + lane * DPB + q * 8) = v;
    }
  }
  loss_block_sums(st, dls, DISTILL ? 0 : L.A, wred, a.stat_part, DISTILL ? nullptr : a.dls_part);  // holds the barriers after step 3

  // ---- 4. dH[s][n] = sum_j dO[s][j] W[j][n], hidden units 32*wave .. +31 (waves beyond HID/32 idle)
  if (wave < NT) {
    bf16x8_t wt[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) wt[ks] = *reinterpret_cast<const bf16x8_t*>(a.wt + (int64_t)(wave * 32 + l32) * HEAD_LD + ks * 16 + h * 8);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      f32x16_t acc;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        const bf16x8_t dv = *reinterpret_cast<const bf16x8_t*>(Da + (t * 32 + l32) * DPA + ks * 16 + h * 8);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wt[ks], dv, acc, 0, 0, 0);
      }
      // acc[g*4+q] = dH[sample t*32 + l32][unit wave*32 + g*8 + h*4 + q]; keep where the activation is positive
      const int sr = t * 32 + l32;
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int nn = wave * 32 + g * 8 + h * 4;
        const uint2 hv = *reinterpret_cast<const uint2*>(Ha + sr * HPA + nn);
        auto pos = [](uint32_t m) -> uint32_t { return (((short)(m & 0xffffu) > 0) ? 0x0000ffffu : 0u) | (((short)(m >> 16) > 0) ? 0xffff0000u : 0u); };
        uint2 o;
        o.x = pack2bf(acc[g * 4], acc[g * 4 + 1]) & pos(hv.x);
        o.y = pack2bf(acc[g * 4 + 2], acc[g * 4 + 3]) & pos(hv.y);
        *reinterpret_cast<uint2*>(DHs + sr * HPA + nn) = o;
      }
    }
  }

  // ---- 5. dW[j][n] partial = sum over the block's samples of dO[s][j] H[s][n]; transposing reads as in k_wgrad
  if (wave < NT) {
    const int g4 = lane >> 4, r16 = lane & 15;
    const int srow = 8 * (g4 >> 1) + (r16 >> 2), scol = 16 * (g4 & 1) + 4 * (r16 & 3);
    f32x16_t acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = 0.f;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const bf16x8_t av = lds_read_tr8(Db + (ks * 16 + srow) * DPB + scol, 4 * DPB);
      const bf16x8_t bv = lds_read_tr8(Hb + (ks * 16 + srow) * HPB + wave * 32 + scol, 4 * HPB);
      acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
    }
    // acc[g*4+q] = dW[j = g*8 + h*4 + q][n = wave*32 + l32]
    float* P = a.wpart + (int64_t)blockIdx.x * a.NH * HID;
#pragma unroll
    for (int e = 0; e < 16; ++e) {
      const int j = (e >> 2) * 8 + h * 4 + (e & 3);
      if (j < a.NH) P[j * HID + wave * 32 + l32] = acc[e];
    }
  }
  if (tid >= 192 && tid - 192 < a.NH) {  // db: column sums of dO in sample order
    const int j = tid - 192;
    float sum = 0.f;
    for (int s = 0; s < 64; ++s) sum += bf2f(Da[s * DPA + j]);
    a.bpart[(int64_t)blockIdx.x * a.NH + j] = sum;
  }
  __syncthreads();
  // ---- dH rows leave as 16-byte segments
  for (int c = tid; c < 64 * CPR; c += 256) {
    const int r = c / CPR, cg = c - r * CPR;
    if (r < ns) *reinterpret_cast<uint4*>(a.dh + (int64_t)(s0 + r) * HID + cg * 8) = *reinterpret_cast<const uint4*>(DHs + r * HPA + cg * 8);
  }
}
