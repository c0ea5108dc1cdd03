// Kernels of the paper's own teacher network (Sec. III-C, Fig. 3) beyond convolutions and linear layers:
// layer normalisation after a convolution (forward with the ReLU, backward with the gain / shift gradients),
// the LSTM cell (forward and backward of one time step for all environments of a chunk; the matrix products
// around it are the library's GEMM kernels), and the small index / state kernels of sequence minibatches.
// Rows of a sequence chunk are time-major: row = t * ne + j for environment j of the chunk's ne environments.
#pragma once
#include "common.hip.h"

#define LN_EPS 1e-5f
#define LN_THREADS 512

// idx[t*ne + j] = t*N + env[j]: the rollout samples of the chunk's environments, time-major.
__global__ void k_seq_index(const int32_t* __restrict__ env, int ne, int T, int N, int32_t* __restrict__ idx) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= ne * T) return;
  const int t = i / ne, j = i - t * ne;
  idx[i] = t * N + env[j];
}

// Block-wide sum of one value per thread in a fixed order (butterfly inside each wave, then the wave sums in
// wave order); every thread gets the result.  red: LN_THREADS / 64 + 1 floats of LDS.
__device__ __forceinline__ float ln_block_sum(float x, float* red) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = x;
  __syncthreads();
  if (threadIdx.x == 0) { float s = 0.f; for (int w = 0; w < nw; ++w) s += red[w]; red[nw] = s; }
  __syncthreads();
  return red[nw];
}

__device__ __forceinline__ void unpack8(const uint4& u, float (&f)[8]) {
  f[0] = bf2f((bf16_t)(u.x & 0xffffu)); f[1] = bf2f((bf16_t)(u.x >> 16));
  f[2] = bf2f((bf16_t)(u.y & 0xffffu)); f[3] = bf2f((bf16_t)(u.y >> 16));
  f[4] = bf2f((bf16_t)(u.z & 0xffffu)); f[5] = bf2f((bf16_t)(u.z >> 16));
  f[6] = bf2f((bf16_t)(u.w & 0xffffu)); f[7] = bf2f((bf16_t)(u.w >> 16));
}

// Layer normalisation + ReLU of convolution outputs.  x: [nimg][m] bf16, channel-last (m = Ho*Wo*C, C a power
// of two >= 8), one block per image walking it three times (sum; squared deviations; normalise) - an image of a
// few hundred KB stays in L2 between the passes.  y[c] = relu(gain[c] * (x - mean) * rstd + shift[c]) goes to the
// image's place in `out` (strides per sample and view), (mean, rstd) to stats[img].
// A thread always meets the same eight channels: LN_THREADS * 8 is a multiple of C.
__global__ __launch_bounds__(LN_THREADS) void k_ln_fwd(const bf16_t* __restrict__ x, int m, int C, const float* __restrict__ gain,
                                                       const float* __restrict__ shift, ImgAddrW out, float2* __restrict__ stats) {
  __shared__ float red[LN_THREADS / 64 + 1];
  const int img = blockIdx.x, tid = threadIdx.x, nch = m >> 3;
  const uint4* xi = reinterpret_cast<const uint4*>(x + (int64_t)img * m);
  float s = 0.f;
  for (int k = tid; k < nch; k += LN_THREADS) { float f[8]; unpack8(xi[k], f); s += ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7])); }
  const float mean = ln_block_sum(s, red) / (float)m;
  float q = 0.f;
  for (int k = tid; k < nch; k += LN_THREADS) {
    float f[8]; unpack8(xi[k], f);
#pragma unroll
    for (int j = 0; j < 8; ++j) { const float d = f[j] - mean; q += d * d; }
  }
  const float rstd = rsqrtf(ln_block_sum(q, red) / (float)m + LN_EPS);
  if (tid == 0) stats[img] = make_float2(mean, rstd);
  const int c0 = (tid * 8) & (C - 1);
  float g[8], b[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { g[j] = gain[c0 + j] * rstd; b[j] = shift[c0 + j] - mean * g[j]; }
  uint4* yo = reinterpret_cast<uint4*>(out.ptr(img));
  for (int k = tid; k < nch; k += LN_THREADS) {
    float f[8]; unpack8(xi[k], f);
    float y[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) y[j] = fmaxf(f[j] * g[j] + b[j], 0.f);
    yo[k] = make_uint4(pack2bf(y[0], y[1]), pack2bf(y[2], y[3]), pack2bf(y[4], y[5]), pack2bf(y[6], y[7]));
  }
}

// Backward of the layer normalisation and of the ReLU behind it.  dy: gradient w.r.t. the rectified output,
// addressed like the forward's output; x, stats: the forward's input and statistics.  The ReLU passes gradient
// where gain[c] xhat + shift[c] > 0 (recomputed here exactly as the forward formed it, so dy may or may not have
// been masked already).  With xhat = (x - mean) rstd and dxhat = dy * gain[c]:  dx = rstd (dxhat - avg(dxhat) - xhat avg(dxhat xhat)),  dgain[c] = sum dy xhat,
// dshift[c] = sum dy.  Block b takes images b, b + gridDim.x, ... and leaves ONE partial [2C] (gain gradients,
// then shift gradients), summed later in block order; all sums in fixed orders.
__global__ __launch_bounds__(LN_THREADS) void k_ln_bwd(ImgAddr dy, const bf16_t* __restrict__ x, const float2* __restrict__ stats, int nimg, int m,
                                                       int C, const float* __restrict__ gain, const float* __restrict__ shift, bf16_t* __restrict__ dx,
                                                       float* __restrict__ partial) {
  __shared__ float red[LN_THREADS / 64 + 1];
  __shared__ float acc[LN_THREADS][17];  // per-thread channel sums (padded rows: conflict-free column walks)
  const int tid = threadIdx.x, nch = m >> 3;
  const int c0 = (tid * 8) & (C - 1);
  float g[8], sh[8], dg[8], db[8];
#pragma unroll
  for (int j = 0; j < 8; ++j) { g[j] = gain[c0 + j]; sh[j] = shift[c0 + j]; dg[j] = 0.f; db[j] = 0.f; }
  for (int img = blockIdx.x; img < nimg; img += gridDim.x) {
    const uint4* xi = reinterpret_cast<const uint4*>(x + (int64_t)img * m);
    const uint4* di = reinterpret_cast<const uint4*>(dy.ptr(img));
    uint4* dxo = reinterpret_cast<uint4*>(dx + (int64_t)img * m);
    const float2 st = stats[img];
    const float mean = st.x, rstd = st.y;
    float s1 = 0.f, s2 = 0.f;
    for (int k = tid; k < nch; k += LN_THREADS) {
      float f[8], d[8]; unpack8(xi[k], f); unpack8(di[k], d);
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float gr = g[j] * rstd, br = sh[j] - mean * gr;   // the forward's y = x * gr + br
        const float dj = (f[j] * gr + br > 0.f) ? d[j] : 0.f;
        const float xh = (f[j] - mean) * rstd, dxh = dj * g[j];
        s1 += dxh; s2 += dxh * xh;
        dg[j] += dj * xh; db[j] += dj;
      }
    }
    const float a1 = ln_block_sum(s1, red) / (float)m;
    const float a2 = ln_block_sum(s2, red) / (float)m;
    for (int k = tid; k < nch; k += LN_THREADS) {
      float f[8], d[8]; unpack8(xi[k], f); unpack8(di[k], d);
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const float gr = g[j] * rstd, br = sh[j] - mean * gr;
        const float dj = (f[j] * gr + br > 0.f) ? d[j] : 0.f;
        const float xh = (f[j] - mean) * rstd;
        o[j] = rstd * (dj * g[j] - a1 - xh * a2);
      }
      dxo[k] = make_uint4(pack2bf(o[0], o[1]), pack2bf(o[2], o[3]), pack2bf(o[4], o[5]), pack2bf(o[6], o[7]));
    }
  }
  __syncthreads();
#pragma unroll
  for (int j = 0; j < 8; ++j) { acc[tid][j] = dg[j]; acc[tid][8 + j] = db[j]; }
  __syncthreads();
  // channel c is held by the threads t with (8 t) mod C = 8 floor(c / 8): t = c/8 + k C/8
  const int groups = C >> 3;
  for (int o = tid; o < 2 * C; o += LN_THREADS) {
    const int c = o < C ? o : o - C, col = (o < C ? 0 : 8) + (c & 7);
    float s = 0.f;
    for (int t = c >> 3; t < LN_THREADS; t += groups) s += acc[t][col];
    partial[(int64_t)blockIdx.x * 2 * C + o] = s;
  }
}

// The forward kernel for images that fit the registers of one 1024-thread block (NCH 16-byte chunks per thread,
// m <= 8192 * NCH): every element is read once instead of three times.  (The backward pass would need both tensors
// in registers, which sixteen waves per block do not have for the larger layers.)
#define LN_RTHREADS 1024
template <int NCH>
__global__ __launch_bounds__(LN_RTHREADS) void k_ln_fwd_reg(const bf16_t* __restrict__ x, int m, int C, const float* __restrict__ gain,
                                                            const float* __restrict__ shift, ImgAddrW out, float2* __restrict__ stats) {
  __shared__ float red[LN_RTHREADS / 64 + 1];
  const int img = blockIdx.x, tid = threadIdx.x, nch = m >> 3;
  const uint4* xi = reinterpret_cast<const uint4*>(x + (int64_t)img * m);
  uint4 v[NCH];
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int k = tid + j * LN_RTHREADS;
    v[j] = k < nch ? xi[k] : make_uint4(0u, 0u, 0u, 0u);
    float f[8]; unpack8(v[j], f);
    s += ((f[0] + f[1]) + (f[2] + f[3])) + ((f[4] + f[5]) + (f[6] + f[7]));
  }
  const float mean = ln_block_sum(s, red) / (float)m;
  float q = 0.f;
#pragma unroll
  for (int j = 0; j < NCH; ++j)
    if (tid + j * LN_RTHREADS < nch) {
      float f[8]; unpack8(v[j], f);
#pragma unroll
      for (int e = 0; e < 8; ++e) { const float d = f[e] - mean; q += d * d; }
    }
  const float rstd = rsqrtf(ln_block_sum(q, red) / (float)m + LN_EPS);
  if (tid == 0) stats[img] = make_float2(mean, rstd);
  const int c0 = (tid * 8) & (C - 1);  // the same for all of a thread's chunks: 8 * LN_RTHREADS is a multiple of C
  float g[8], b[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) { g[e] = gain[c0 + e] * rstd; b[e] = shift[c0 + e] - mean * g[e]; }
  uint4* yo = reinterpret_cast<uint4*>(out.ptr(img));
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int k = tid + j * LN_RTHREADS;
    if (k < nch) {
      float f[8]; unpack8(v[j], f);
      float y[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) y[e] = fmaxf(f[e] * g[e] + b[e], 0.f);
      yo[k] = make_uint4(pack2bf(y[0], y[1]), pack2bf(y[2], y[3]), pack2bf(y[4], y[5]), pack2bf(y[6], y[7]));
    }
  }
}

// State that enters the first step of the chunk's environments: h (as bf16, into the h columns of row block 0 of
// the layer's input matrix xh [rows][ld], columns [col_h, col_h + H)) and c (fp32, c_enter row block 0), gathered
// from the per-environment initial states h0 / c0 [N][H] of this layer.
__global__ void k_lstm_init(const int32_t* __restrict__ env, int ne, int H, const float* __restrict__ h0, const float* __restrict__ c0,
                            bf16_t* __restrict__ xh, int64_t ld, int col_h, float* __restrict__ c_enter) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= ne * H) return;
  const int j = i / H, k = i - j * H;
  const int64_t e = env[j];
  xh[(int64_t)j * ld + col_h + k] = f2bf(h0[e * H + k]);
  c_enter[i] = c0[e * H + k];
}

__device__ __forceinline__ float sigmoidf_(float x) { return 1.f / (1.f + __expf(-x)); }

// LSTM cell of one time step for the chunk's ne environments (Hochreiter & Schmidhuber; gate order i, f, g, o).
// pre [ne][4H]: W_ih x + W_hh h_enter + b from the GEMM.  Writes the gate activations (fp32, kept for the backward
// pass), h = o tanh(f c_enter + i g) as bf16 into the next layer's input row (or the trunk's input) `h_out`, and the
// state that enters the NEXT step - zero where this step's done flag is set - into h_next (bf16, may be NULL at the
// last step) and c_next (fp32).  idx_t: the rollout sample numbers of this step's rows (for the done flags).
__global__ void k_lstm_cell_fwd(int ne, int H, const float* __restrict__ pre, const float* __restrict__ c_enter, const uint8_t* __restrict__ done,
                                const int32_t* __restrict__ idx_t, float* __restrict__ gates, bf16_t* __restrict__ h_out, int64_t ld_out,
                                bf16_t* __restrict__ h_next, int64_t ld_next, float* __restrict__ c_next) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= ne * H) return;
  const int j = i / H, k = i - j * H;
  const float* p = pre + (int64_t)j * 4 * H;
  const float ig = sigmoidf_(p[k]), fg = sigmoidf_(p[H + k]), gg = tanhf(p[2 * H + k]), og = sigmoidf_(p[3 * H + k]);
  float* go = gates + (int64_t)j * 4 * H;
  go[k] = ig; go[H + k] = fg; go[2 * H + k] = gg; go[3 * H + k] = og;
  const float c = fg * c_enter[i] + ig * gg;
  const bf16_t h = f2bf(og * tanhf(c));
  h_out[(int64_t)j * ld_out + k] = h;
  const bool reset = done[idx_t[j]] != 0;
  if (h_next) h_next[(int64_t)j * ld_next + k] = reset ? (bf16_t)0 : h;
  if (c_next) c_next[i] = reset ? 0.f : c;
}

// Backward of that cell.  dh_above [ne][.]: gradient w.r.t. h_t from the layer above (or the trunk); dh_rec
// (NULL at the last step): gradient w.r.t. the state that entered step t+1, from that step's GEMM; dc_carry
// [ne][H] fp32: gradient w.r.t. the cell state that entered step t+1 (in) / step t (out).  Both recurrent terms
// are dropped where this step's done flag reset the state.  Writes the gate pre-activation gradients da [ne][4H]
// (bf16: the operand of the two GEMMs that follow).
__global__ void k_lstm_cell_bwd(int ne, int H, const float* __restrict__ gates, const float* __restrict__ c_enter, const uint8_t* __restrict__ done,
                                const int32_t* __restrict__ idx_t, const bf16_t* __restrict__ dh_above, int64_t ld_above,
                                const bf16_t* __restrict__ dh_rec, int64_t ld_rec, float* __restrict__ dc_carry, int first_carry,
                                bf16_t* __restrict__ da) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= ne * H) return;
  const int j = i / H, k = i - j * H;
  const bool cut = done[idx_t[j]] != 0;
  float dh = bf2f(dh_above[(int64_t)j * ld_above + k]);
  float dc_in = 0.f;
  if (!cut && !first_carry) {
    if (dh_rec) dh += bf2f(dh_rec[(int64_t)j * ld_rec + k]);
    dc_in = dc_carry[i];
  }
  const float* go = gates + (int64_t)j * 4 * H;
  const float ig = go[k], fg = go[H + k], gg = go[2 * H + k], og = go[3 * H + k], ce = c_enter[i];
  const float tc = tanhf(fg * ce + ig * gg);
  const float dc = dh * og * (1.f - tc * tc) + dc_in;
  bf16_t* d = da + (int64_t)j * 4 * H;
  d[k] = f2bf(dc * gg * ig * (1.f - ig));
  d[H + k] = f2bf(dc * ce * fg * (1.f - fg));
  d[2 * H + k] = f2bf(dc * ig * (1.f - gg * gg));
  d[3 * H + k] = f2bf(dh * tc * og * (1.f - og));
  dc_carry[i] = dc * fg;
}

// d[r][0..cols) = 0 where x[r][0..cols) <= 0 (rows of stride ld_d / ld_x): the ReLU mask of a stored activation
// applied to its gradient when the kernel that produced the gradient could not (eight elements per thread).
__global__ void k_mask_rows(int64_t rows, int cols, bf16_t* __restrict__ d, int64_t ld_d, const bf16_t* __restrict__ x, int64_t ld_x) {
  const int cpr = cols >> 3;
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * cpr) return;
  const int64_t r = i / cpr;
  const int k = (int)(i - r * cpr) * 8;
  uint4 v = *reinterpret_cast<const uint4*>(d + r * ld_d + k);
  const uint4 m = *reinterpret_cast<const uint4*>(x + r * ld_x + k);
  auto keep = [](uint32_t w) -> uint32_t { return (((short)(w & 0xffffu) > 0) ? 0x0000ffffu : 0u) | (((short)(w >> 16) > 0) ? 0xffff0000u : 0u); };
  v.x &= keep(m.x); v.y &= keep(m.y); v.z &= keep(m.z); v.w &= keep(m.w);
  *reinterpret_cast<uint4*>(d + r * ld_d + k) = v;
}
