/*
 * CPU oracle for the PPO learner path: GAE, minibatch permutation, the
 * depth-CNN + MLP actor-critic forward/backward, the clipped-PPO and
 * distillation losses, and Adam.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 statement of
 * what the learner computes, used only by the tests, the smoke check and the
 * benchmark's cpu_baseline leg.  It shares no code with the HIP library and
 * the product path never calls it.
 *
 * What the paper fixes and what it leaves open: the paper's learner appends
 * (obs, actions, rew, done) once per step to a trajectory buffer and then
 * calls TrainPPO on it (Algorithm 2); it trains "end-to-end with PPO"
 * (Sec. III-C) and distils into a stereo-RGB student by supervising the
 * student's actions with the teacher's output (Sec. I, Sec. III-C).  It
 * prints no formula for GAE, the PPO loss or Adam; the formulas below are
 * the standard definitions from the PPO / GAE / Adam papers it relies on.
 * Every function below names the definition it writes out.
 *
 * Pins (tests/test_oracle_*.py): GAE closed forms at lambda=0 and lambda=1
 * and a brute-force double sum; convolution and linear layers against a
 * library routine and tap-count closed forms; the whole forward/loss/backward
 * against fp64 automatic differentiation and central finite differences;
 * loss closed forms at ratio=1; Adam against closed forms and a library
 * optimiser; permutation bijection / brute force / published SplitMix64
 * vectors; the policy step against a library normal density, the closed
 * form at zero noise and the ratio-1 property of the loss on its own
 * output.  The composed multi-minibatch update (orc_ppo_update,
 * orc_distill_update) is pinned only transitively through those parts:
 * parity unpinned by the paper for the composed loop.
 *
 * Layouts (all row-major):
 *   obs      float  [B][n_views][in_c][in_h][in_w]
 *   proprio  double [B][P]        action double [B][A]
 *   params   double, canonical order:
 *       for each conv l: W[Co][Ci][k][k], b[Co]
 *       for each fc   l: W[out][in], b[out]      (in of fc0 = n_views*flat + P,
 *                                                 flat in (c,h,w) order)
 *       head:  W_mu[A][h], b_mu[A]
 *       if has_value_head: w_v[h], b_v, logstd[A]
 *   (the full order with the optional layer-norm, embedding, LSTM and auxiliary-head
 *    parameters is given at make_geom)
 *
 * Pins of the recurrent teacher's parts and of the auxiliary MLP head (tests/test_oracle_pins.py):
 * layer normalisation against a library group normalisation, the LSTM against a library LSTM module
 * (forward, final state, gradients through time), state resets at done flags against a sequence cut
 * by hand, the whole recurrent forward/loss/backward against fp64 automatic differentiation and
 * central finite differences, the auxiliary head against automatic differentiation.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_MAX_LAYERS 8

typedef struct {
  int32_t n_views, in_c, in_h, in_w;
  int32_t proprio_dim, act_dim;
  int32_t n_conv, conv_ch[ORC_MAX_LAYERS], conv_k, conv_stride, conv_pad;
  int32_t n_fc, fc_dim[ORC_MAX_LAYERS];
  int32_t has_value_head;
  /* the deployed student's extra MLP head (Sec. IV-C): with aux_hidden > 0 the last aux_dim output
   * columns come from  W_a2 relu(W_a1 h + b_a1) + b_a2  on the last hidden layer h instead of the
   * linear mean head (which then has act_dim - aux_dim rows) */
  int32_t aux_hidden, aux_dim;
  /* the paper's own teacher (Sec. III-C, Fig. 3): layer normalisation after every convolution,
   * a linear embedding of each view's flattened features, LSTM layers between the concatenation
   * with the proprioception and the MLP */
  int32_t layer_norm, embed_dim, lstm_layers, lstm_units;
} orc_net;

typedef struct {
  double clip_eps, vclip_eps /* <=0: off */, vf_coef, ent_coef;
  double aux_coef;  /* distillation: weight of the auxiliary columns' error */
  int32_t aux_dim;  /* distillation: the last aux_dim head columns are the auxiliary output; 0: none */
} orc_loss_cfg;

typedef struct {
  double lr, beta1, beta2, eps;
  double max_grad_norm; /* <= 0: no clipping */
  double desired_kl;    /* > 0: KL-adaptive learning rate (PPO only), see update_loop */
  double lr_min, lr_max;
} orc_adam_cfg;

/* stats slots */
enum { ST_PI = 0, ST_V, ST_ENT, ST_KL, ST_CLIPFRAC, ST_GNORM, ST_TOTAL, ST_LR, ST_N };

/* ------------------------------------------------------------------ */
/* geometry                                                            */
/* ------------------------------------------------------------------ */
static int conv_out(int in, int k, int s, int p) { return (in + 2 * p - k) / s + 1; }

#define ORC_MAX_LSTM 4
typedef struct {
  int n_conv, n_fc, nl, H;
  int c[ORC_MAX_LAYERS + 1], h[ORC_MAX_LAYERS + 1], w[ORC_MAX_LAYERS + 1];
  int fc_in[ORC_MAX_LAYERS + 1], fc_out[ORC_MAX_LAYERS + 1];
  int lstm_in[ORC_MAX_LSTM];
  int64_t convW[ORC_MAX_LAYERS], convB[ORC_MAX_LAYERS], lnG[ORC_MAX_LAYERS], lnB[ORC_MAX_LAYERS];
  int64_t embW, embB;
  int64_t lstmWih[ORC_MAX_LSTM], lstmWhh[ORC_MAX_LSTM], lstmB[ORC_MAX_LSTM];
  int64_t fcW[ORC_MAX_LAYERS], fcB[ORC_MAX_LAYERS];
  int64_t muW, muB, vW, vB, logstd, a1W, a1B, a2W, a2B, total;
  int flat, enc, feat, trunk_in, hid, A_main;
} geom;

/* Canonical parameter order: for each conv l: W, b, [LN gain[Co], LN shift[Co]]; [embedding W[E][flat], b[E]];
 * for each LSTM layer: W_ih[4H][in], W_hh[4H][H], b[4H] (gate order i, f, g, o); for each hidden layer W, b;
 * mean head W[A_main][h], b; [value head w[h], b; logstd[A]]; [aux head W_a1[X][h], b_a1, W_a2[aux_dim][X], b_a2]. */
static void make_geom(const orc_net *n, geom *g) {
  g->n_conv = n->n_conv; g->n_fc = n->n_fc; g->nl = n->lstm_layers; g->H = n->lstm_units;
  g->c[0] = n->in_c; g->h[0] = n->in_h; g->w[0] = n->in_w;
  int64_t off = 0;
  for (int l = 0; l < n->n_conv; ++l) {
    g->c[l + 1] = n->conv_ch[l];
    g->h[l + 1] = conv_out(g->h[l], n->conv_k, n->conv_stride, n->conv_pad);
    g->w[l + 1] = conv_out(g->w[l], n->conv_k, n->conv_stride, n->conv_pad);
    g->convW[l] = off; off += (int64_t)g->c[l + 1] * g->c[l] * n->conv_k * n->conv_k;
    g->convB[l] = off; off += g->c[l + 1];
    g->lnG[l] = g->lnB[l] = -1;
    if (n->layer_norm) { g->lnG[l] = off; off += g->c[l + 1]; g->lnB[l] = off; off += g->c[l + 1]; }
  }
  g->flat = g->c[n->n_conv] * g->h[n->n_conv] * g->w[n->n_conv];
  g->embW = g->embB = -1; g->enc = g->flat;
  if (n->embed_dim > 0) { g->enc = n->embed_dim; g->embW = off; off += (int64_t)n->embed_dim * g->flat; g->embB = off; off += n->embed_dim; }
  int in = n->n_views * g->enc + n->proprio_dim;
  g->feat = in;
  for (int l = 0; l < g->nl; ++l) {
    g->lstm_in[l] = in;
    g->lstmWih[l] = off; off += (int64_t)4 * g->H * in;
    g->lstmWhh[l] = off; off += (int64_t)4 * g->H * g->H;
    g->lstmB[l] = off; off += 4 * g->H;
    in = g->H;
  }
  g->trunk_in = in;
  for (int l = 0; l < n->n_fc; ++l) {
    g->fc_in[l] = in; g->fc_out[l] = n->fc_dim[l];
    g->fcW[l] = off; off += (int64_t)in * n->fc_dim[l];
    g->fcB[l] = off; off += n->fc_dim[l];
    in = n->fc_dim[l];
  }
  g->hid = in;
  g->A_main = n->act_dim - (n->aux_hidden > 0 ? n->aux_dim : 0);
  g->muW = off; off += (int64_t)g->A_main * in;
  g->muB = off; off += g->A_main;
  g->vW = g->vB = g->logstd = -1;
  if (n->has_value_head) {
    g->vW = off; off += in;
    g->vB = off; off += 1;
    g->logstd = off; off += n->act_dim;
  }
  g->a1W = g->a1B = g->a2W = g->a2B = -1;
  if (n->aux_hidden > 0) {
    g->a1W = off; off += (int64_t)n->aux_hidden * in;
    g->a1B = off; off += n->aux_hidden;
    g->a2W = off; off += (int64_t)n->aux_dim * n->aux_hidden;
    g->a2B = off; off += n->aux_dim;
  }
  g->total = off;
}

int64_t orc_param_count(const orc_net *n) { geom g; make_geom(n, &g); return g.total; }
int32_t orc_flat_dim(const orc_net *n) { geom g; make_geom(n, &g); return g.flat; }

/* Image bytes held by an experience buffer of N envs x T steps
 * (Sec. III-B sizing example: envs * steps * pixels * bytes per element). */
int64_t orc_buffer_image_bytes(int64_t N, int64_t T, int64_t n_views, int64_t c, int64_t h,
                               int64_t w, int64_t elem_bytes) {
  return N * T * n_views * c * h * w * elem_bytes;
}

/* float -> bfloat16 (round to nearest, ties to even) -> float. */
float orc_bf16_rne(float x) {
  uint32_t u; memcpy(&u, &x, 4);
  if ((u & 0x7fffffffu) > 0x7f800000u) { u |= 0x00400000u; u &= 0xffff0000u; }
  else { uint32_t lsb = (u >> 16) & 1u; u += 0x7fffu + lsb; u &= 0xffff0000u; }
  float y; memcpy(&y, &u, 4); return y;
}

/* Operand-precision mode of the network arithmetic.
 *   0: exact  - everything in fp64 (the definition).
 *   1: bf16 operands - the arithmetic "bf16 matrix operands, wide accumulation": every STORED
 *      activation (images, ReLU outputs, proprioception), every stored activation-gradient
 *      (loss gradients w.r.t. the head outputs, each layer's masked input gradient) and the
 *      weight matrix of every layer are rounded once to bf16 (RNE); biases, log-std, all sums
 *      and the loss stay wide.
 * Mode 1 exists because the discrete decisions of the method (ReLU masks, which branch of the
 * clipped surrogate / clipped value loss is active) must be taken in the same precision on both
 * sides of a comparison; it changes no formula. */
static int g_quant = 0;
void orc_set_quant(int32_t mode) { g_quant = mode; }
int32_t orc_get_quant(void) { return g_quant; }
static double q(double x) { return g_quant ? (double)orc_bf16_rne((float)x) : x; }

/* ------------------------------------------------------------------ */
/* GAE (Schulman et al., generalized advantage estimation), per env,   */
/* reverse in time.  The done flag of step t belongs to the transition */
/* taken at t (Algorithm 1: obs, rew, dones come from one Env.Step), so */
/* it masks the bootstrap from t+1.                                    */
/*   delta_t = r_t + gamma*(1-d_t)*V_{t+1} - V_t                        */
/*   A_t     = delta_t + gamma*lambda*(1-d_t)*A_{t+1},  A_T = 0         */
/*   R_t     = A_t + V_t,   V_T = last_value                            */
/* arrays are [T][N].                                                  */
/* ------------------------------------------------------------------ */
void orc_gae(int32_t T, int32_t N, const double *reward, const uint8_t *done, const double *value,
             const double *last_value, double gamma, double lambda, double *adv, double *ret) {
  for (int n = 0; n < N; ++n) {
    double next_v = last_value[n], next_a = 0.0;
    for (int t = T - 1; t >= 0; --t) {
      int64_t i = (int64_t)t * N + n;
      double nt = done[i] ? 0.0 : 1.0;
      double delta = reward[i] + gamma * next_v * nt - value[i];
      double a = delta + gamma * lambda * nt * next_a;
      adv[i] = a; ret[i] = a + value[i];
      next_a = a; next_v = value[i];
    }
  }
}

/* ------------------------------------------------------------------ */
/* Minibatch permutation: indices 0..S-1 sorted by (key_i, i), with    */
/* key_i = SplitMix64 finaliser (Steele, Lea, Flood 2014; Vigna's      */
/* public-domain splitmix64) applied to a per-(seed, update, epoch)    */
/* stream base plus (i+1) golden-gamma increments.                     */
/* ------------------------------------------------------------------ */
static uint64_t sm64_finalise(uint64_t z) {
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ULL;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBULL;
  return z ^ (z >> 31);
}
/* n-th output (n = 0,1,...) of a SplitMix64 generator whose state starts at `state`. */
uint64_t orc_splitmix64_nth(uint64_t state, uint64_t n) {
  return sm64_finalise(state + (n + 1) * 0x9E3779B97F4A7C15ULL);
}
uint64_t orc_perm_stream(uint64_t seed, uint64_t update, uint64_t epoch) {
  /* stream base: hash the (seed, update, epoch) triple by chaining the finaliser */
  uint64_t s = sm64_finalise(seed + 0x9E3779B97F4A7C15ULL);
  s = sm64_finalise(s ^ (update + 0x9E3779B97F4A7C15ULL));
  s = sm64_finalise(s ^ (epoch + 0x9E3779B97F4A7C15ULL));
  return s;
}
uint64_t orc_perm_key(uint64_t seed, uint64_t update, uint64_t epoch, uint64_t i) {
  return orc_splitmix64_nth(orc_perm_stream(seed, update, epoch), i);
}
typedef struct { uint64_t key; int32_t idx; } keyidx;
static int cmp_keyidx(const void *a, const void *b) {
  const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
  if (x->key != y->key) return x->key < y->key ? -1 : 1;
  return x->idx < y->idx ? -1 : (x->idx > y->idx);
}
void orc_permutation(uint64_t seed, uint64_t update, uint64_t epoch, int64_t S, int32_t *out) {
  keyidx *a = (keyidx *)malloc(sizeof(keyidx) * (size_t)(S > 0 ? S : 1));
  for (int64_t i = 0; i < S; ++i) { a[i].key = orc_perm_key(seed, update, epoch, (uint64_t)i); a[i].idx = (int32_t)i; }
  qsort(a, (size_t)S, sizeof(keyidx), cmp_keyidx);
  for (int64_t i = 0; i < S; ++i) out[i] = a[i].idx;
  free(a);
}

/* ------------------------------------------------------------------ */
/* Layers, written from their definitions.                             */
/* conv: cross-correlation, zero padding,                              */
/*   y[co][i][j] = b[co] + sum_{ci,u,v} W[co][ci][u][v] x[ci][s*i+u-p][s*j+v-p] */
/* ------------------------------------------------------------------ */
static void conv_fwd(const double *x, int ci_n, int H, int W, const double *w, const double *b,
                     int co_n, int k, int s, int p, double *y, int Ho, int Wo) {
  for (int co = 0; co < co_n; ++co)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        double acc = b[co];
        for (int ci = 0; ci < ci_n; ++ci)
          for (int u = 0; u < k; ++u) {
            int iy = s * i + u - p;
            if (iy < 0 || iy >= H) continue;
            for (int v = 0; v < k; ++v) {
              int ix = s * j + v - p;
              if (ix < 0 || ix >= W) continue;
              acc += w[((co * ci_n + ci) * k + u) * k + v] * x[(ci * H + iy) * W + ix];
            }
          }
        y[(co * Ho + i) * Wo + j] = acc;
      }
}
/* adjoint of conv_fwd: accumulates dW, db and (if dx != NULL) dx from dy */
static void conv_bwd(const double *x, int ci_n, int H, int W, const double *w, int co_n, int k,
                     int s, int p, const double *dy, int Ho, int Wo, double *dw, double *db,
                     double *dx) {
  for (int co = 0; co < co_n; ++co)
    for (int i = 0; i < Ho; ++i)
      for (int j = 0; j < Wo; ++j) {
        double g = dy[(co * Ho + i) * Wo + j];
        if (g == 0.0) continue;
        db[co] += g;
        for (int ci = 0; ci < ci_n; ++ci)
          for (int u = 0; u < k; ++u) {
            int iy = s * i + u - p;
            if (iy < 0 || iy >= H) continue;
            for (int v = 0; v < k; ++v) {
              int ix = s * j + v - p;
              if (ix < 0 || ix >= W) continue;
              int wi = ((co * ci_n + ci) * k + u) * k + v, xi = (ci * H + iy) * W + ix;
              dw[wi] += g * x[xi];
              if (dx) dx[xi] += g * w[wi];
            }
          }
      }
}
static void lin_fwd(const double *x, int in, const double *w, const double *b, int out, double *y) {
  for (int o = 0; o < out; ++o) {
    double acc = b ? b[o] : 0.0;
    for (int i = 0; i < in; ++i) acc += w[(int64_t)o * in + i] * x[i];
    y[o] = acc;
  }
}
static void lin_bwd(const double *x, int in, const double *w, int out, const double *dy, double *dw,
                    double *db, double *dx) {
  for (int o = 0; o < out; ++o) {
    double g = dy[o];
    if (db) db[o] += g;
    for (int i = 0; i < in; ++i) {
      dw[(int64_t)o * in + i] += g * x[i];
      if (dx) dx[i] += g * w[(int64_t)o * in + i];
    }
  }
}

/* ------------------------------------------------------------------ */
/* Layer normalisation of one convolution output (Ba, Kiros, Hinton     */
/* 2016), statistics over all C*H*W values of one sample, gain and      */
/* shift per channel:                                                   */
/*   mean = avg(x), var = avg((x-mean)^2)  (population variance)        */
/*   xhat = (x - mean) / sqrt(var + 1e-5),  y[c][.] = g[c] xhat + b[c]  */
/* ------------------------------------------------------------------ */
#define ORC_LN_EPS 1e-5
static void ln_fwd(const double *x, int C, int HW, const double *gain, const double *shift, double *xhat,
                   double *rstd_out, double *y) {
  int64_t m = (int64_t)C * HW;
  double mean = 0, var = 0;
  for (int64_t i = 0; i < m; ++i) mean += x[i];
  mean /= (double)m;
  for (int64_t i = 0; i < m; ++i) var += (x[i] - mean) * (x[i] - mean);
  var /= (double)m;
  double rstd = 1.0 / sqrt(var + ORC_LN_EPS);
  for (int c = 0; c < C; ++c)
    for (int k = 0; k < HW; ++k) {
      int64_t i = (int64_t)c * HW + k;
      xhat[i] = (x[i] - mean) * rstd;
      y[i] = gain[c] * xhat[i] + shift[c];
    }
  *rstd_out = rstd;
}
/* adjoint of ln_fwd: dgain, dshift accumulate; dx = rstd (dxhat - avg(dxhat) - xhat avg(dxhat xhat)) */
static void ln_bwd(const double *dy, const double *xhat, double rstd, int C, int HW, const double *gain,
                   double *dgain, double *dshift, double *dx) {
  int64_t m = (int64_t)C * HW;
  double s1 = 0, s2 = 0;
  for (int c = 0; c < C; ++c)
    for (int k = 0; k < HW; ++k) {
      int64_t i = (int64_t)c * HW + k;
      dgain[c] += dy[i] * xhat[i];
      dshift[c] += dy[i];
      double dxh = dy[i] * gain[c];
      s1 += dxh; s2 += dxh * xhat[i];
    }
  s1 /= (double)m; s2 /= (double)m;
  for (int c = 0; c < C; ++c)
    for (int k = 0; k < HW; ++k) {
      int64_t i = (int64_t)c * HW + k;
      dx[i] = rstd * (dy[i] * gain[c] - s1 - xhat[i] * s2);
    }
}

static double sigmoid(double x) { return 1.0 / (1.0 + exp(-x)); }

/* activations of ONE time step of one environment */
typedef struct {
  double *conv[4][ORC_MAX_LAYERS + 1];  /* per view: input image (l = 0), then each layer's output after ReLU */
  double *xhat[4][ORC_MAX_LAYERS + 1];  /* with layer_norm: normalised conv output of layer l-1 at index l */
  double rstd[4][ORC_MAX_LAYERS + 1];
  double *feat;                         /* [views*enc + P]: encoder outputs, then proprioception */
  double *gate[ORC_MAX_LSTM];           /* [4H]: i, f, g, o after their nonlinearities */
  double *cell[ORC_MAX_LSTM], *hid[ORC_MAX_LSTM], *tcell[ORC_MAX_LSTM];  /* c_t, h_t, tanh(c_t) */
  double *cin[ORC_MAX_LSTM], *hin[ORC_MAX_LSTM];                         /* the state that entered the step */
  double *fc[ORC_MAX_LAYERS];           /* hidden activations after ReLU */
  double *aux;                          /* [aux_hidden] after ReLU */
  double *mu; double v;                 /* outputs: [A] (aux head's columns last), value */
} acts;

typedef struct {  /* gradient scratch of one environment (reused by every step) */
  double *dconv[ORC_MAX_LAYERS + 1], *dpre;
  double *dfeat, *dfc[ORC_MAX_LAYERS], *daux, *dtrunk;
  double *dx[ORC_MAX_LSTM + 1];  /* gradient w.r.t. the input of LSTM layer l; [nl] = w.r.t. the top output */
  double *da;                    /* [4H] gate pre-activation gradients */
  double *dh_next[ORC_MAX_LSTM], *dc_next[ORC_MAX_LSTM];  /* from step t+1 into (h_t, c_t) */
  double *tmp;                   /* conv scratch */
} grads_ws;

static double *dalloc(int64_t n) { return (double *)calloc((size_t)(n > 0 ? n : 1), sizeof(double)); }

static void acts_alloc(const orc_net *n, const geom *g, acts *a) {
  memset(a, 0, sizeof *a);
  for (int v = 0; v < n->n_views; ++v)
    for (int l = 0; l <= n->n_conv; ++l) {
      a->conv[v][l] = dalloc((int64_t)g->c[l] * g->h[l] * g->w[l]);
      if (n->layer_norm && l > 0) a->xhat[v][l] = dalloc((int64_t)g->c[l] * g->h[l] * g->w[l]);
    }
  a->feat = dalloc(g->feat);
  for (int l = 0; l < g->nl; ++l) {
    a->gate[l] = dalloc(4 * g->H); a->cell[l] = dalloc(g->H); a->hid[l] = dalloc(g->H); a->tcell[l] = dalloc(g->H);
    a->cin[l] = dalloc(g->H); a->hin[l] = dalloc(g->H);
  }
  for (int l = 0; l < n->n_fc; ++l) a->fc[l] = dalloc(g->fc_out[l]);
  a->aux = dalloc(n->aux_hidden);
  a->mu = dalloc(n->act_dim);
}
static void acts_free(const orc_net *n, const geom *g, acts *a) {
  for (int v = 0; v < n->n_views; ++v)
    for (int l = 0; l <= n->n_conv; ++l) { free(a->conv[v][l]); free(a->xhat[v][l]); }
  free(a->feat);
  for (int l = 0; l < g->nl; ++l) { free(a->gate[l]); free(a->cell[l]); free(a->hid[l]); free(a->tcell[l]); free(a->cin[l]); free(a->hin[l]); }
  for (int l = 0; l < n->n_fc; ++l) free(a->fc[l]);
  free(a->aux); free(a->mu);
}
static void ws_alloc(const orc_net *n, const geom *g, grads_ws *w) {
  memset(w, 0, sizeof *w);
  int64_t mx = 0;
  for (int l = 0; l <= n->n_conv; ++l) {
    int64_t m = (int64_t)g->c[l] * g->h[l] * g->w[l];
    w->dconv[l] = dalloc(m);
    if (m > mx) mx = m;
  }
  w->dpre = dalloc(mx); w->tmp = dalloc(mx);
  w->dfeat = dalloc(g->feat); w->dtrunk = dalloc(g->trunk_in); w->daux = dalloc(n->aux_hidden);
  for (int l = 0; l < n->n_fc; ++l) w->dfc[l] = dalloc(g->fc_out[l]);
  for (int l = 0; l <= g->nl; ++l) w->dx[l] = dalloc(l < g->nl ? g->lstm_in[l] : g->H);
  w->da = dalloc(4 * g->H);
  for (int l = 0; l < g->nl; ++l) { w->dh_next[l] = dalloc(g->H); w->dc_next[l] = dalloc(g->H); }
}
static void ws_free(const orc_net *n, const geom *g, grads_ws *w) {
  for (int l = 0; l <= n->n_conv; ++l) free(w->dconv[l]);
  free(w->dpre); free(w->tmp); free(w->dfeat); free(w->dtrunk); free(w->daux);
  for (int l = 0; l < n->n_fc; ++l) free(w->dfc[l]);
  for (int l = 0; l <= g->nl; ++l) free(w->dx[l]);
  free(w->da);
  for (int l = 0; l < g->nl; ++l) { free(w->dh_next[l]); free(w->dc_next[l]); }
}

/* Forward of one time step of one environment.
 *   encoder, per view with shared weights: conv (+bias) [-> layer norm] -> ReLU, ..., flatten in (c,h,w)
 *     order [-> linear embedding, no activation];
 *   features = [encoder(view 0), encoder(view 1), ..., proprioception];
 *   LSTM layers (Hochreiter & Schmidhuber; gate order i, f, g, o):
 *     a = W_ih x + W_hh h_in + b;  i, f, o = sigmoid(a_i, a_f, a_o);  g = tanh(a_g);
 *     c = f c_in + i g;  h = o tanh(c);   (h_in, c_in) given by the caller in a->hin / a->cin;
 *   hidden layers (+bias, ReLU); linear mean head (no squashing), scalar value head; with aux_hidden > 0 the
 *   last aux_dim outputs are W_a2 relu(W_a1 h + b_a1) + b_a2. */
static void step_forward(const orc_net *n, const geom *g, const double *P, const float *obs,
                         const double *proprio, acts *a) {
  for (int v = 0; v < n->n_views; ++v) {
    int64_t px = (int64_t)g->c[0] * g->h[0] * g->w[0];
    for (int64_t i = 0; i < px; ++i) a->conv[v][0][i] = q((double)obs[v * px + i]);  /* the stored image */
    for (int l = 0; l < n->n_conv; ++l) {
      double *y = a->conv[v][l + 1];
      conv_fwd(a->conv[v][l], g->c[l], g->h[l], g->w[l], P + g->convW[l], P + g->convB[l],
               g->c[l + 1], n->conv_k, n->conv_stride, n->conv_pad, y, g->h[l + 1], g->w[l + 1]);
      int64_t m = (int64_t)g->c[l + 1] * g->h[l + 1] * g->w[l + 1];
      if (n->layer_norm) {
        for (int64_t i = 0; i < m; ++i) y[i] = q(y[i]);  /* the stored convolution output */
        ln_fwd(y, g->c[l + 1], g->h[l + 1] * g->w[l + 1], P + g->lnG[l], P + g->lnB[l], a->xhat[v][l + 1],
               &a->rstd[v][l + 1], y);
      }
      for (int64_t i = 0; i < m; ++i) y[i] = (y[i] > 0.0) ? q(y[i]) : 0.0;
    }
    if (n->embed_dim > 0) {
      double *e = a->feat + (size_t)v * g->enc;
      lin_fwd(a->conv[v][n->n_conv], g->flat, P + g->embW, P + g->embB, g->enc, e);
      for (int i = 0; i < g->enc; ++i) e[i] = q(e[i]);
    } else {
      memcpy(a->feat + (size_t)v * g->flat, a->conv[v][n->n_conv], sizeof(double) * (size_t)g->flat);
    }
  }
  for (int i = 0; i < n->proprio_dim; ++i) a->feat[n->n_views * g->enc + i] = q(proprio[i]);
  const double *x = a->feat;
  const int H = g->H;
  for (int l = 0; l < g->nl; ++l) {
    double *ga = a->gate[l];
    lin_fwd(x, g->lstm_in[l], P + g->lstmWih[l], P + g->lstmB[l], 4 * H, ga);
    for (int r = 0; r < 4 * H; ++r) {
      double acc = 0;
      for (int k = 0; k < H; ++k) acc += P[g->lstmWhh[l] + (int64_t)r * H + k] * a->hin[l][k];
      ga[r] += acc;
    }
    for (int k = 0; k < H; ++k) {
      double ig = sigmoid(ga[k]), fg = sigmoid(ga[H + k]), gg = tanh(ga[2 * H + k]), og = sigmoid(ga[3 * H + k]);
      ga[k] = ig; ga[H + k] = fg; ga[2 * H + k] = gg; ga[3 * H + k] = og;
      a->cell[l][k] = fg * a->cin[l][k] + ig * gg;
      a->tcell[l][k] = tanh(a->cell[l][k]);
      a->hid[l][k] = q(og * a->tcell[l][k]);
    }
    x = a->hid[l];
  }
  for (int l = 0; l < n->n_fc; ++l) {
    lin_fwd(x, g->fc_in[l], P + g->fcW[l], P + g->fcB[l], g->fc_out[l], a->fc[l]);
    for (int i = 0; i < g->fc_out[l]; ++i) a->fc[l][i] = (a->fc[l][i] > 0.0) ? q(a->fc[l][i]) : 0.0;
    x = a->fc[l];
  }
  lin_fwd(x, g->hid, P + g->muW, P + g->muB, g->A_main, a->mu);
  a->v = 0.0;
  if (n->has_value_head) lin_fwd(x, g->hid, P + g->vW, P + g->vB, 1, &a->v);
  if (n->aux_hidden > 0) {
    lin_fwd(x, g->hid, P + g->a1W, P + g->a1B, n->aux_hidden, a->aux);
    for (int i = 0; i < n->aux_hidden; ++i) a->aux[i] = (a->aux[i] > 0.0) ? q(a->aux[i]) : 0.0;
    lin_fwd(a->aux, n->aux_hidden, P + g->a2W, P + g->a2B, n->aux_dim, a->mu + g->A_main);
  }
}

/* Backward of one time step from dmu[A], dv and (recurrent nets) the gradients w->dh_next / w->dc_next that
 * step t+1 sent into this step's (h, c); accumulates into G (parameter layout) and leaves in w->dh_next /
 * w->dc_next the gradients w.r.t. the state that ENTERED this step.  ReLU passes gradient where the stored
 * activation is > 0. */
static void step_backward(const orc_net *n, const geom *g, const double *P, acts *a, grads_ws *w,
                          const double *dmu, double dv, double *G) {
  const double *x = n->n_fc ? a->fc[n->n_fc - 1] : (g->nl ? a->hid[g->nl - 1] : a->feat);
  double *dx = n->n_fc ? w->dfc[n->n_fc - 1] : w->dtrunk;
  memset(dx, 0, sizeof(double) * (size_t)g->hid);
  lin_bwd(x, g->hid, P + g->muW, g->A_main, dmu, G + g->muW, G + g->muB, dx);
  if (n->has_value_head) lin_bwd(x, g->hid, P + g->vW, 1, &dv, G + g->vW, G + g->vB, dx);
  if (n->aux_hidden > 0) {
    memset(w->daux, 0, sizeof(double) * (size_t)n->aux_hidden);
    lin_bwd(a->aux, n->aux_hidden, P + g->a2W, n->aux_dim, dmu + g->A_main, G + g->a2W, G + g->a2B, w->daux);
    for (int i = 0; i < n->aux_hidden; ++i) w->daux[i] = (a->aux[i] > 0.0) ? q(w->daux[i]) : 0.0;
    lin_bwd(x, g->hid, P + g->a1W, n->aux_hidden, w->daux, G + g->a1W, G + g->a1B, dx);
  }
  for (int l = n->n_fc - 1; l >= 0; --l) {
    double *dy = w->dfc[l];
    for (int i = 0; i < g->fc_out[l]; ++i) dy[i] = (a->fc[l][i] > 0.0) ? q(dy[i]) : 0.0;
    const double *xin = l ? a->fc[l - 1] : (g->nl ? a->hid[g->nl - 1] : a->feat);
    double *dxin = l ? w->dfc[l - 1] : w->dtrunk;
    memset(dxin, 0, sizeof(double) * (size_t)g->fc_in[l]);
    lin_bwd(xin, g->fc_in[l], P + g->fcW[l], g->fc_out[l], dy, G + g->fcW[l], G + g->fcB[l], dxin);
  }
  /* w->dtrunk = gradient w.r.t. the trunk's input: the features, or the top LSTM layer's h */
  double *dfeat = w->dtrunk;
  if (g->nl > 0) {
    const int H = g->H;
    memcpy(w->dx[g->nl], w->dtrunk, sizeof(double) * (size_t)H);
    for (int l = g->nl - 1; l >= 0; --l) {
      const double *ga = a->gate[l];
      const double *xin = l ? a->hid[l - 1] : a->feat;
      for (int k = 0; k < H; ++k) {
        double dh = q(w->dx[l + 1][k] + w->dh_next[l][k]);  /* the stored gradient w.r.t. h_t */
        double ig = ga[k], fg = ga[H + k], gg = ga[2 * H + k], og = ga[3 * H + k], tc = a->tcell[l][k];
        double dc = dh * og * (1.0 - tc * tc) + w->dc_next[l][k];
        w->da[k] = dc * gg * ig * (1.0 - ig);
        w->da[H + k] = dc * a->cin[l][k] * fg * (1.0 - fg);
        w->da[2 * H + k] = dc * ig * (1.0 - gg * gg);
        w->da[3 * H + k] = dh * tc * og * (1.0 - og);
        w->dc_next[l][k] = dc * fg;
      }
      for (int r = 0; r < 4 * H; ++r) w->da[r] = q(w->da[r]);
      memset(w->dx[l], 0, sizeof(double) * (size_t)g->lstm_in[l]);
      lin_bwd(xin, g->lstm_in[l], P + g->lstmWih[l], 4 * H, w->da, G + g->lstmWih[l], G + g->lstmB[l], w->dx[l]);
      memset(w->dh_next[l], 0, sizeof(double) * (size_t)H);
      lin_bwd(a->hin[l], H, P + g->lstmWhh[l], 4 * H, w->da, G + g->lstmWhh[l], NULL, w->dh_next[l]);
    }
    dfeat = w->dx[0];
  }
  for (int v = 0; v < n->n_views; ++v) {
    int L = n->n_conv;
    if (n->embed_dim > 0) {
      double *de = dfeat + (size_t)v * g->enc;
      for (int i = 0; i < g->enc; ++i) de[i] = q(de[i]);
      memset(w->dconv[L], 0, sizeof(double) * (size_t)g->flat);
      lin_bwd(a->conv[v][L], g->flat, P + g->embW, g->enc, de, G + g->embW, G + g->embB, w->dconv[L]);
    } else {
      memcpy(w->dconv[L], dfeat + (size_t)v * g->flat, sizeof(double) * (size_t)g->flat);
    }
    for (int l = L - 1; l >= 0; --l) {
      int64_t m = (int64_t)g->c[l + 1] * g->h[l + 1] * g->w[l + 1];
      double *dy = w->dconv[l + 1];
      for (int64_t i = 0; i < m; ++i) dy[i] = (a->conv[v][l + 1][i] > 0.0) ? q(dy[i]) : 0.0;
      if (n->layer_norm) {
        ln_bwd(dy, a->xhat[v][l + 1], a->rstd[v][l + 1], g->c[l + 1], g->h[l + 1] * g->w[l + 1], P + g->lnG[l],
               G + g->lnG[l], G + g->lnB[l], w->dpre);
        for (int64_t i = 0; i < m; ++i) w->dpre[i] = q(w->dpre[i]);  /* the stored gradient w.r.t. the convolution output */
        dy = w->dpre;
      }
      double *dxl = l ? w->dconv[l] : NULL;
      if (dxl) memset(dxl, 0, sizeof(double) * (size_t)g->c[l] * g->h[l] * g->w[l]);
      conv_bwd(a->conv[v][l], g->c[l], g->h[l], g->w[l], P + g->convW[l], g->c[l + 1], n->conv_k,
               n->conv_stride, n->conv_pad, dy, g->h[l + 1], g->w[l + 1],
               G + g->convW[l], G + g->convB[l], dxl);
    }
  }
}

/* Copy of the parameters as the layers use them: in bf16-operand mode the weight matrices of
 * every layer are rounded to bf16; everything else (biases, log-std, layer-norm gain and shift) is unchanged. */
static double *operand_params(const orc_net *n, const geom *g, const double *params) {
  double *P = (double *)malloc(sizeof(double) * (size_t)g->total);
  memcpy(P, params, sizeof(double) * (size_t)g->total);
  if (!g_quant) return P;
  for (int l = 0; l < n->n_conv; ++l)
    for (int64_t i = g->convW[l]; i < g->convB[l]; ++i) P[i] = q(P[i]);
  if (n->embed_dim > 0) for (int64_t i = g->embW; i < g->embB; ++i) P[i] = q(P[i]);
  for (int l = 0; l < g->nl; ++l)
    for (int64_t i = g->lstmWih[l]; i < g->lstmB[l]; ++i) P[i] = q(P[i]);
  for (int l = 0; l < n->n_fc; ++l)
    for (int64_t i = g->fcW[l]; i < g->fcB[l]; ++i) P[i] = q(P[i]);
  for (int64_t i = g->muW; i < g->muB; ++i) P[i] = q(P[i]);
  if (n->has_value_head)
    for (int64_t i = g->vW; i < g->vB; ++i) P[i] = q(P[i]);
  if (n->aux_hidden > 0) {
    for (int64_t i = g->a1W; i < g->a1B; ++i) P[i] = q(P[i]);
    for (int64_t i = g->a2W; i < g->a2B; ++i) P[i] = q(P[i]);
  }
  return P;
}

/* The state that enters step t of environment b: the given initial state at t = 0 (zero when none is given),
 * else the state step t-1 left, or zero when that step ended the episode (its done flag is set: Algorithm 1
 * returns obs, rew, dones from one Env.Step, so done_{t-1} says that the observation of step t starts a new
 * episode). */
static void enter_state(const geom *g, int64_t Benv, int64_t b, int t, const uint8_t *done, const double *h0,
                        const double *c0, const acts *prev, acts *cur) {
  for (int l = 0; l < g->nl; ++l)
    for (int k = 0; k < g->H; ++k) {
      double h = 0, c = 0;
      if (t == 0) {
        if (h0) h = h0[((int64_t)l * Benv + b) * g->H + k];
        if (c0) c = c0[((int64_t)l * Benv + b) * g->H + k];
      } else if (!(done && done[(int64_t)(t - 1) * Benv + b])) { h = prev->hid[l][k]; c = prev->cell[l][k]; }
      cur->hin[l][k] = h; cur->cin[l][k] = c;
    }
}

/* Network outputs for Benv environments x L steps, arrays time-major ([L][Benv]...): mu [L][Benv][A], v [L][Benv]
 * (v untouched without a value head).  Feed-forward nets (lstm_layers = 0) treat every (t, b) independently;
 * recurrent nets carry (h, c) along t from (h0, c0) [layers][Benv][H] (NULL: zeros) with resets at done flags
 * (done [L][Benv], NULL: none) and return the final state in hT, cT when those are not NULL. */
void orc_seq_forward(const orc_net *n, const double *params_in, int64_t Benv, int32_t L, const float *obs,
                     const double *proprio, const uint8_t *done, const double *h0, const double *c0,
                     double *mu, double *v, double *hT, double *cT) {
  geom g; make_geom(n, &g);
  double *params = operand_params(n, &g, params_in);
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
#pragma omp parallel
  {
    acts a[2]; acts_alloc(n, &g, &a[0]); acts_alloc(n, &g, &a[1]);
#pragma omp for schedule(static)
    for (int64_t b = 0; b < Benv; ++b) {
      for (int t = 0; t < L; ++t) {
        acts *cur = &a[t & 1], *prev = &a[(t & 1) ^ 1];
        int64_t s = (int64_t)t * Benv + b;
        enter_state(&g, Benv, b, t, done, h0, c0, prev, cur);
        step_forward(n, &g, params, obs + s * obs_sz, proprio + s * n->proprio_dim, cur);
        memcpy(mu + s * n->act_dim, cur->mu, sizeof(double) * (size_t)n->act_dim);
        if (n->has_value_head) v[s] = cur->v;
      }
      const acts *last = &a[(L - 1) & 1];
      for (int l = 0; l < g.nl; ++l)
        for (int k = 0; k < g.H; ++k) {
          if (hT) hT[((int64_t)l * Benv + b) * g.H + k] = last->hid[l][k];
          if (cT) cT[((int64_t)l * Benv + b) * g.H + k] = last->cell[l][k];
        }
    }
    acts_free(n, &g, &a[0]); acts_free(n, &g, &a[1]);
  }
  free(params);
}

/* Network outputs for B independent samples: mu [B][A], v [B]. */
void orc_forward(const orc_net *n, const double *params_in, int64_t B, const float *obs,
                 const double *proprio, double *mu, double *v) {
  orc_seq_forward(n, params_in, B, 1, obs, proprio, NULL, NULL, NULL, mu, v, NULL, NULL);
}

/* ------------------------------------------------------------------ */
/* Policy step of the collection loop (Algorithm 2: the policy maps the */
/* stacked observations to actions, and the record is appended after    */
/* the simulators have stepped).  Diagonal Gaussian policy:             */
/*   a_j   = mu_j + exp(logsigma_j) * xi_j,   xi given by the caller    */
/*   logp  = sum_j [-((a_j-mu_j)/sigma_j)^2/2 - logsigma_j - ln(2pi)/2] */
/*   value = V(obs)                                                     */
/* logp is evaluated at the action, the way the loss evaluates it       */
/* later, so that the first pass over fresh data sees ratio 1.          */
/* Outputs: action [B][A], logp [B], value [B].                         */
/* ------------------------------------------------------------------ */
void orc_act(const orc_net *n, const double *params, int64_t B, const float *obs,
             const double *proprio, const double *noise, double *action, double *logp,
             double *value) {
  const double LN2PI = 1.8378770664093454835606594728112;
  geom g; make_geom(n, &g);
  const int A = n->act_dim;
  const double *logstd = params + g.logstd;
  double *mu = (double *)malloc(sizeof(double) * (size_t)B * A);
  orc_forward(n, params, B, obs, proprio, mu, value);
  for (int64_t s = 0; s < B; ++s) {
    double lp = 0;
    for (int j = 0; j < A; ++j) {
      double sg = exp(logstd[j]);
      double a = mu[s * A + j] + sg * noise[s * A + j];
      double z = (a - mu[s * A + j]) / sg;
      action[s * A + j] = a;
      lp += -0.5 * z * z - logstd[j] - 0.5 * LN2PI;
    }
    logp[s] = lp;
  }
  free(mu);
}

/* ------------------------------------------------------------------ */
/* Clipped-PPO loss on network outputs (Schulman et al. 2017, eq. 7     */
/* and 9), diagonal Gaussian policy with state-independent log-std.    */
/*   logp = sum_j [-((a-mu)/sigma)^2/2 - logsigma - ln(2pi)/2]         */
/*   rho  = exp(logp - logp_old)                                       */
/*   L_pi = -mean min(rho*A, clip(rho,1-e,1+e)*A)                      */
/*   L_V  = mean (V-R)^2, or with clipping                             */
/*          mean max((V-R)^2, (V_old+clip(V-V_old,-ev,ev)-R)^2)        */
/*   H    = sum_j (logsigma_j + ln(2 pi e)/2)                          */
/*   L    = L_pi + c_v L_V - c_e H                                     */
/* Outputs: stats[ST_*] (ST_GNORM untouched), and if non-NULL the      */
/* gradients dmu[B][A], dv[B], dlogstd[A] of L.                        */
/* ------------------------------------------------------------------ */
void orc_ppo_loss(int64_t B, int32_t A, const double *mu, const double *v, const double *logstd,
                  const double *action, const double *logp_old, const double *v_old,
                  const double *adv, const double *ret, const orc_loss_cfg *cfg, double *stats,
                  double *dmu, double *dv, double *dlogstd) {
  const double LN2PI = 1.8378770664093454835606594728112;
  double lpi = 0, lv = 0, kl = 0, cf = 0, ent = 0;
  for (int j = 0; j < A; ++j) ent += logstd[j] + 0.5 * (LN2PI + 1.0);
  if (dlogstd) for (int j = 0; j < A; ++j) dlogstd[j] = -cfg->ent_coef;
  double invB = 1.0 / (double)B, e = cfg->clip_eps;
  for (int64_t s = 0; s < B; ++s) {
    double logp = 0;
    for (int j = 0; j < A; ++j) {
      double z = (action[s * A + j] - mu[s * A + j]) / exp(logstd[j]);
      logp += -0.5 * z * z - logstd[j] - 0.5 * LN2PI;
    }
    double lr = logp - logp_old[s], rho = exp(lr), a = adv[s];
    double rc = rho < 1 - e ? 1 - e : (rho > 1 + e ? 1 + e : rho);
    double s1 = rho * a, s2 = rc * a;
    lpi += -(s1 < s2 ? s1 : s2);
    /* the unclipped term carries the gradient when it is the minimum (ties: unclipped) */
    double dlogp = (s1 <= s2) ? -invB * a * rho : 0.0;
    kl += (rho - 1.0) - lr;
    cf += (fabs(rho - 1.0) > e) ? 1.0 : 0.0;
    double dvs, err = v[s] - ret[s];
    if (cfg->vclip_eps > 0) {
      double ev = cfg->vclip_eps, d = v[s] - v_old[s];
      double dc = d < -ev ? -ev : (d > ev ? ev : d);
      double errc = v_old[s] + dc - ret[s];
      if (errc * errc > err * err) {
        lv += errc * errc;
        dvs = (d >= -ev && d <= ev) ? 2.0 * errc : 0.0;
      } else { lv += err * err; dvs = 2.0 * err; }
    } else { lv += err * err; dvs = 2.0 * err; }
    if (dv) dv[s] = cfg->vf_coef * invB * dvs;
    if (dmu)
      for (int j = 0; j < A; ++j) {
        double sg = exp(logstd[j]), z = (action[s * A + j] - mu[s * A + j]) / sg;
        dmu[s * A + j] = dlogp * z / sg;
        dlogstd[j] += dlogp * (z * z - 1.0);
      }
  }
  stats[ST_PI] = lpi * invB; stats[ST_V] = lv * invB; stats[ST_ENT] = ent;
  stats[ST_KL] = kl * invB; stats[ST_CLIPFRAC] = cf * invB;
  stats[ST_TOTAL] = stats[ST_PI] + cfg->vf_coef * stats[ST_V] - cfg->ent_coef * ent;
}

/* Distillation loss.  Without auxiliary columns: mean over batch and action dims of
 * (pred - teacher)^2.  With the last X = aux_dim columns an auxiliary output (the deployed
 * student's object position, Sec. IV-C; the paper gives no weighting):
 *   L = mean_b [ 1/(A-X) sum_{j<A-X} e_bj^2 ] + aux_coef * mean_b [ 1/X sum_{j>=A-X} e_bj^2 ],
 * the two means reported as stats[ST_PI] and stats[ST_V]. */
void orc_mse_loss(int64_t B, int32_t A, int32_t aux_dim, double aux_coef, const double *pred,
                  const double *target, double *stats, double *dpred) {
  int Aa = A - aux_dim;
  double la = 0, lx = 0;
  double sa = 1.0 / ((double)B * Aa), sx = aux_dim > 0 ? aux_coef / ((double)B * aux_dim) : 0.0;
  for (int64_t b = 0; b < B; ++b)
    for (int j = 0; j < A; ++j) {
      double d = pred[b * A + j] - target[b * A + j];
      if (j < Aa) la += d * d; else lx += d * d;
      if (dpred) dpred[b * A + j] = 2.0 * (j < Aa ? sa : sx) * d;
    }
  for (int i = 0; i < ST_N; ++i) stats[i] = 0;
  stats[ST_PI] = la * sa;
  stats[ST_V] = aux_dim > 0 ? lx / ((double)B * aux_dim) : 0.0;
  stats[ST_TOTAL] = stats[ST_PI] + (aux_dim > 0 ? aux_coef * stats[ST_V] : 0.0);
}

/* One minibatch of Benv environments x L steps (time-major arrays; L = 1 for feed-forward nets, where an
 * "environment" is just a sample): forward everything, evaluate the loss on all Benv*L outputs (its means
 * run over all of them), backward everything.  Recurrent nets: back-propagation through time over the L steps
 * of each environment, the state gradient cut where a done flag reset the state. */
static void minibatch_grad(const orc_net *n, const double *params_in, int64_t Benv, int32_t L, const float *obs,
                           const double *proprio, const double *action, const double *logp_old,
                           const double *v_old, const double *adv, const double *ret, const uint8_t *done,
                           const double *h0, const double *c0,
                           const orc_loss_cfg *cfg, int distill, double *grads, double *stats) {
  geom g; make_geom(n, &g);
  int A = n->act_dim;
  int64_t B = Benv * L;
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
  double *mu = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *v = (double *)calloc((size_t)B, sizeof(double));
  double *dmu = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *dv = (double *)calloc((size_t)B, sizeof(double));
  double *params = operand_params(n, &g, params_in);
  orc_seq_forward(n, params_in, Benv, L, obs, proprio, done, h0, c0, mu, v, NULL, NULL);
  memset(grads, 0, sizeof(double) * (size_t)g.total);
  if (distill) orc_mse_loss(B, A, cfg ? cfg->aux_dim : 0, cfg ? cfg->aux_coef : 0.0, mu, action, stats, dmu);
  else
    orc_ppo_loss(B, A, mu, v, params + g.logstd, action, logp_old, v_old, adv, ret, cfg, stats,
                 dmu, dv, grads + g.logstd);
  /* the loss gradients w.r.t. the head outputs are stored activations-gradients */
  for (int64_t i = 0; i < B * A; ++i) dmu[i] = q(dmu[i]);
  for (int64_t i = 0; i < B; ++i) dv[i] = q(dv[i]);
  int nth = 1;
#ifdef _OPENMP
  nth = omp_get_max_threads();
#endif
  double *tg = (double *)calloc((size_t)nth * (size_t)g.total, sizeof(double));
#pragma omp parallel
  {
    int tid = 0;
#ifdef _OPENMP
    tid = omp_get_thread_num();
#endif
    acts *a = (acts *)malloc(sizeof(acts) * (size_t)L);
    for (int t = 0; t < L; ++t) acts_alloc(n, &g, &a[t]);
    grads_ws w; ws_alloc(n, &g, &w);
    double *G = tg + (size_t)tid * (size_t)g.total;
#pragma omp for schedule(static)
    for (int64_t b = 0; b < Benv; ++b) {
      for (int t = 0; t < L; ++t) {
        int64_t s = (int64_t)t * Benv + b;
        enter_state(&g, Benv, b, t, done, h0, c0, t ? &a[t - 1] : NULL, &a[t]);
        step_forward(n, &g, params, obs + s * obs_sz, proprio + s * n->proprio_dim, &a[t]);
      }
      for (int l = 0; l < g.nl; ++l) {
        memset(w.dh_next[l], 0, sizeof(double) * (size_t)g.H);
        memset(w.dc_next[l], 0, sizeof(double) * (size_t)g.H);
      }
      for (int t = L - 1; t >= 0; --t) {
        int64_t s = (int64_t)t * Benv + b;
        step_backward(n, &g, params, &a[t], &w, dmu + s * A, dv[s], G);
        /* what is left in dh_next / dc_next goes to step t-1, unless step t started a new episode */
        if (t > 0 && done && done[(int64_t)(t - 1) * Benv + b])
          for (int l = 0; l < g.nl; ++l) {
            memset(w.dh_next[l], 0, sizeof(double) * (size_t)g.H);
            memset(w.dc_next[l], 0, sizeof(double) * (size_t)g.H);
          }
      }
    }
    for (int t = 0; t < L; ++t) acts_free(n, &g, &a[t]);
    free(a);
    ws_free(n, &g, &w);
  }
  for (int t = 0; t < nth; ++t)
    for (int64_t i = 0; i < g.total; ++i) grads[i] += tg[(size_t)t * (size_t)g.total + i];
  double gn = 0;
  for (int64_t i = 0; i < g.total; ++i) gn += grads[i] * grads[i];
  stats[ST_GNORM] = sqrt(gn);
  free(tg); free(mu); free(v); free(dmu); free(dv); free(params);
}

/* Loss, stats and parameter gradients of the PPO objective on one minibatch of B independent samples. */
void orc_ppo_loss_grad(const orc_net *n, const double *params, int64_t B, const float *obs,
                       const double *proprio, const double *action, const double *logp_old,
                       const double *v_old, const double *adv, const double *ret,
                       const orc_loss_cfg *cfg, double *grads, double *stats) {
  minibatch_grad(n, params, B, 1, obs, proprio, action, logp_old, v_old, adv, ret, NULL, NULL, NULL, cfg, 0, grads, stats);
}
/* The same on a minibatch of Benv whole sequences of L steps (time-major arrays), for recurrent nets. */
void orc_seq_ppo_loss_grad(const orc_net *n, const double *params, int64_t Benv, int32_t L, const float *obs,
                           const double *proprio, const double *action, const double *logp_old,
                           const double *v_old, const double *adv, const double *ret, const uint8_t *done,
                           const double *h0, const double *c0, const orc_loss_cfg *cfg, double *grads,
                           double *stats) {
  minibatch_grad(n, params, Benv, L, obs, proprio, action, logp_old, v_old, adv, ret, done, h0, c0, cfg, 0, grads, stats);
}
void orc_distill_loss_grad(const orc_net *n, const double *params, int64_t B, const float *obs,
                           const double *proprio, const double *teacher, int32_t aux_dim,
                           double aux_coef, double *grads, double *stats) {
  orc_loss_cfg lc; memset(&lc, 0, sizeof lc); lc.aux_dim = aux_dim; lc.aux_coef = aux_coef;
  minibatch_grad(n, params, B, 1, obs, proprio, teacher, NULL, NULL, NULL, NULL, NULL, NULL, NULL, &lc, 1, grads, stats);
}

/* Adam (Kingma & Ba 2015, Algorithm 1), epsilon added to the bias-corrected
 * root: m = b1 m + (1-b1) g; v = b2 v + (1-b2) g^2;
 * theta -= lr * (m/(1-b1^k)) / (sqrt(v/(1-b2^k)) + eps), k = 1,2,... */
void orc_adam_step(int64_t n, double *params, double *m, double *v, const double *grads, int64_t k,
                   const orc_adam_cfg *c) {
  double c1 = 1.0 - pow(c->beta1, (double)k), c2 = 1.0 - pow(c->beta2, (double)k);
  for (int64_t i = 0; i < n; ++i) {
    m[i] = c->beta1 * m[i] + (1.0 - c->beta1) * grads[i];
    v[i] = c->beta2 * v[i] + (1.0 - c->beta2) * grads[i] * grads[i];
    params[i] -= c->lr * (m[i] / c1) / (sqrt(v[i] / c2) + c->eps);
  }
}

/* Global gradient-norm clipping (Pascanu et al. 2013, as the common deep-learning
 * libraries implement it): with n = ||g||_2 over ALL parameters, g <- g * min(1, c / (n + 1e-6)).
 * Returns n, the norm before clipping.  max_norm <= 0: g untouched. */
double orc_clip_grad_norm(int64_t n, double *grads, double max_norm) {
  double sq = 0;
  for (int64_t i = 0; i < n; ++i) sq += grads[i] * grads[i];
  double norm = sqrt(sq);
  if (max_norm > 0) {
    double coef = max_norm / (norm + 1e-6);
    if (coef < 1.0)
      for (int64_t i = 0; i < n; ++i) grads[i] *= coef;
  }
  return norm;
}

/* Advantage normalisation over the whole rollout (all S = N*T samples, once per update):
 *   out = (adv - mean) / (std + 1e-8),  std = population standard deviation. */
void orc_normalize_adv(int64_t S, const double *adv, double *out) {
  double mean = 0, var = 0;
  for (int64_t i = 0; i < S; ++i) mean += adv[i];
  mean /= (double)S;
  for (int64_t i = 0; i < S; ++i) var += (adv[i] - mean) * (adv[i] - mean);
  double sd = sqrt(var / (double)S);
  for (int64_t i = 0; i < S; ++i) out[i] = (adv[i] - mean) / (sd + 1e-8);
}

/* One learner update over a rollout of N environments x T steps (arrays [T][N]..., flat sample s = t*N + n).
 * Feed-forward nets: for each epoch draw a fresh permutation of the S = N*T samples, split it into
 * `minibatches` contiguous chunks, and for each chunk: forward, loss, backward, one Adam step.
 * Recurrent nets (lstm_layers > 0): the unit of a minibatch is a whole environment (the LSTM is unrolled over
 * the T steps of the horizon, Sec. III-B/III-C), so the permutation is over the N environments, a minibatch is
 * N/minibatches environments x all T steps, the initial state of each environment is (h0, c0)
 * [layers][N][H] (NULL: zeros), and done flags reset the state (see enter_state).
 * adv/ret/logp_old/v_old stay fixed for the whole update.  *step is the Adam step counter (in/out).
 * With ac->max_grad_norm > 0 the gradient is clipped to that global norm before the Adam step
 * (the grad-norm statistic stays the norm before clipping).
 * With ac->desired_kl > 0 (PPO only) the learning rate follows the divergence between the behaviour
 * policy and the current one, measured on each minibatch before its step by the sample estimate
 * kl = mean((rho - 1) - log rho) the loss already reports: kl > 2 desired_kl divides the rate by 1.5
 * (not below lr_min), kl < desired_kl / 2 multiplies it by 1.5 (not above lr_max); the new rate is the
 * one this minibatch's Adam step uses and the next minibatch starts from.  The paper names no
 * schedule; this is the usual one of on-policy robot-learning code, with the sampled estimate in
 * place of the closed-form Gaussian divergence.  stats[.][ST_LR] is the rate each step used.
 * stats: [epochs*minibatches][ST_N]; grads_last: gradients of the last minibatch. */
static void update_loop(const orc_net *n, double *params, double *m, double *v, int64_t *step,
                        int64_t N, int32_t T, const float *obs, const double *proprio, const double *action,
                        const double *logp_old, const double *v_old, const double *adv,
                        const double *ret, const uint8_t *done, const double *h0, const double *c0,
                        const orc_loss_cfg *lc, const orc_adam_cfg *ac,
                        int32_t epochs, int32_t minibatches, uint64_t seed, uint64_t update_idx,
                        int distill, double *stats, double *grads_last) {
  geom g; make_geom(n, &g);
  int A = n->act_dim, P = n->proprio_dim;
  const int recurrent = g.nl > 0;
  const int64_t S = N * T;
  const int64_t U = recurrent ? N : S;   /* units the permutation shuffles */
  const int32_t L = recurrent ? T : 1;   /* steps per unit */
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
  int64_t Bu = U / minibatches, B = Bu * L;
  int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)U);
  float *mobs = (float *)malloc(sizeof(float) * (size_t)B * (size_t)obs_sz);
  double *mpro = (double *)malloc(sizeof(double) * (size_t)B * P);
  double *mact = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *mlp = (double *)calloc((size_t)B, sizeof(double)), *mvo = (double *)calloc((size_t)B, sizeof(double));
  double *mad = (double *)calloc((size_t)B, sizeof(double)), *mre = (double *)calloc((size_t)B, sizeof(double));
  uint8_t *mdo = (uint8_t *)calloc((size_t)B, 1);
  double *mh0 = (double *)calloc((size_t)(g.nl * Bu * g.H + 1), sizeof(double));
  double *mc0 = (double *)calloc((size_t)(g.nl * Bu * g.H + 1), sizeof(double));
  double *grads = (double *)malloc(sizeof(double) * (size_t)g.total);
  orc_adam_cfg cur = *ac;
  for (int e = 0; e < epochs; ++e) {
    orc_permutation(seed, update_idx, (uint64_t)e, U, perm);
    for (int mb = 0; mb < minibatches; ++mb) {
      for (int64_t b = 0; b < Bu; ++b) {
        int64_t u = perm[(int64_t)mb * Bu + b];
        for (int t = 0; t < L; ++t) {
          int64_t s = recurrent ? (int64_t)t * N + u : u;  /* source sample */
          int64_t d = (int64_t)t * Bu + b;                  /* slot in the time-major minibatch */
          memcpy(mobs + d * obs_sz, obs + s * obs_sz, sizeof(float) * (size_t)obs_sz);
          memcpy(mpro + d * P, proprio + s * P, sizeof(double) * (size_t)P);
          memcpy(mact + d * A, action + s * A, sizeof(double) * (size_t)A);
          if (!distill) { mlp[d] = logp_old[s]; mvo[d] = v_old[s]; mad[d] = adv[s]; mre[d] = ret[s]; }
          if (recurrent) mdo[d] = done ? done[s] : 0;
        }
        for (int l = 0; l < g.nl; ++l)
          for (int k = 0; k < g.H; ++k) {
            mh0[((int64_t)l * Bu + b) * g.H + k] = h0 ? h0[((int64_t)l * N + u) * g.H + k] : 0.0;
            mc0[((int64_t)l * Bu + b) * g.H + k] = c0 ? c0[((int64_t)l * N + u) * g.H + k] : 0.0;
          }
      }
      double *st = stats + ((int64_t)e * minibatches + mb) * ST_N;
      minibatch_grad(n, params, Bu, L, mobs, mpro, mact, mlp, mvo, mad, mre, recurrent ? mdo : NULL,
                     recurrent ? mh0 : NULL, recurrent ? mc0 : NULL, lc, distill, grads, st);
      *step += 1;
      /* the gradient reported for the last minibatch is the one before clipping */
      if (grads_last && e == epochs - 1 && mb == minibatches - 1)
        memcpy(grads_last, grads, sizeof(double) * (size_t)g.total);
      if (!distill && ac->desired_kl > 0) {
        double kl = st[ST_KL];
        if (kl > 2.0 * ac->desired_kl) cur.lr = fmax(ac->lr_min, cur.lr / 1.5);
        else if (kl < 0.5 * ac->desired_kl) cur.lr = fmin(ac->lr_max, cur.lr * 1.5);
      }
      st[ST_LR] = cur.lr;
      orc_clip_grad_norm(g.total, grads, ac->max_grad_norm);
      orc_adam_step(g.total, params, m, v, grads, *step, &cur);
    }
  }
  free(perm); free(mobs); free(mpro); free(mact); free(mlp); free(mvo); free(mad); free(mre); free(mdo);
  free(mh0); free(mc0); free(grads);
}

/* Feed-forward nets: S flat samples (the rollout's [T][N] arrays flattened). */
void orc_ppo_update(const orc_net *n, double *params, double *m, double *v, int64_t *step, int64_t S,
                    const float *obs, const double *proprio, const double *action,
                    const double *logp_old, const double *v_old, const double *adv,
                    const double *ret, const orc_loss_cfg *lc, const orc_adam_cfg *ac,
                    int32_t epochs, int32_t minibatches, uint64_t seed, uint64_t update_idx,
                    double *stats, double *grads_last) {
  update_loop(n, params, m, v, step, S, 1, obs, proprio, action, logp_old, v_old, adv, ret, NULL, NULL, NULL, lc, ac,
              epochs, minibatches, seed, update_idx, 0, stats, grads_last);
}
/* Any net, rollout given as [T][N] arrays; recurrent nets need this form. */
void orc_seq_ppo_update(const orc_net *n, double *params, double *m, double *v, int64_t *step, int64_t N, int32_t T,
                        const float *obs, const double *proprio, const double *action,
                        const double *logp_old, const double *v_old, const double *adv,
                        const double *ret, const uint8_t *done, const double *h0, const double *c0,
                        const orc_loss_cfg *lc, const orc_adam_cfg *ac,
                        int32_t epochs, int32_t minibatches, uint64_t seed, uint64_t update_idx,
                        double *stats, double *grads_last) {
  update_loop(n, params, m, v, step, N, T, obs, proprio, action, logp_old, v_old, adv, ret, done, h0, c0, lc, ac,
              epochs, minibatches, seed, update_idx, 0, stats, grads_last);
}
void orc_distill_update(const orc_net *n, double *params, double *m, double *v, int64_t *step,
                        int64_t S, const float *obs, const double *proprio, const double *teacher,
                        int32_t aux_dim, double aux_coef,
                        const orc_adam_cfg *ac, int32_t epochs, int32_t minibatches, uint64_t seed,
                        uint64_t update_idx, double *stats, double *grads_last) {
  orc_loss_cfg lc; memset(&lc, 0, sizeof lc); lc.aux_dim = aux_dim; lc.aux_coef = aux_coef;
  update_loop(n, params, m, v, step, S, 1, obs, proprio, teacher, NULL, NULL, NULL, NULL, NULL, NULL, NULL, &lc, ac,
              epochs, minibatches, seed, update_idx, 1, stats, grads_last);
}

/* Number of threads the sample loops use from now on (timing aid of the benchmark's baseline leg). */
void orc_set_num_threads(int32_t n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

int32_t orc_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}
