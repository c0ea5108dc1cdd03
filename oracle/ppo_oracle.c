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

typedef struct {
  int n_conv, n_fc;
  int c[ORC_MAX_LAYERS + 1], h[ORC_MAX_LAYERS + 1], w[ORC_MAX_LAYERS + 1];
  int fc_in[ORC_MAX_LAYERS + 1], fc_out[ORC_MAX_LAYERS + 1];
  int64_t convW[ORC_MAX_LAYERS], convB[ORC_MAX_LAYERS];
  int64_t fcW[ORC_MAX_LAYERS], fcB[ORC_MAX_LAYERS];
  int64_t muW, muB, vW, vB, logstd, total;
  int flat, feat, hid;
} geom;

static void make_geom(const orc_net *n, geom *g) {
  g->n_conv = n->n_conv; g->n_fc = n->n_fc;
  g->c[0] = n->in_c; g->h[0] = n->in_h; g->w[0] = n->in_w;
  int64_t off = 0;
  for (int l = 0; l < n->n_conv; ++l) {
    g->c[l + 1] = n->conv_ch[l];
    g->h[l + 1] = conv_out(g->h[l], n->conv_k, n->conv_stride, n->conv_pad);
    g->w[l + 1] = conv_out(g->w[l], n->conv_k, n->conv_stride, n->conv_pad);
    g->convW[l] = off; off += (int64_t)g->c[l + 1] * g->c[l] * n->conv_k * n->conv_k;
    g->convB[l] = off; off += g->c[l + 1];
  }
  g->flat = g->c[n->n_conv] * g->h[n->n_conv] * g->w[n->n_conv];
  int in = n->n_views * g->flat + n->proprio_dim;
  g->feat = in;
  for (int l = 0; l < n->n_fc; ++l) {
    g->fc_in[l] = in; g->fc_out[l] = n->fc_dim[l];
    g->fcW[l] = off; off += (int64_t)in * n->fc_dim[l];
    g->fcB[l] = off; off += n->fc_dim[l];
    in = n->fc_dim[l];
  }
  g->hid = in;
  g->muW = off; off += (int64_t)n->act_dim * in;
  g->muB = off; off += n->act_dim;
  g->vW = g->vB = g->logstd = -1;
  if (n->has_value_head) {
    g->vW = off; off += in;
    g->vB = off; off += 1;
    g->logstd = off; off += n->act_dim;
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

/* per-sample activation storage */
typedef struct {
  /* conv activations per view: act[v][l] for l = 0..n_conv (0 = input image), post-ReLU */
  double *conv[4][ORC_MAX_LAYERS + 1];
  double *feat;                       /* fc0 input: [views*flat + P] */
  double *fc[ORC_MAX_LAYERS];         /* post-ReLU hidden activations */
  double *mu; double v;
  /* gradient scratch */
  double *dconv[ORC_MAX_LAYERS + 1];
  double *dfeat; double *dfc[ORC_MAX_LAYERS];
} acts;

static void acts_alloc(const orc_net *n, const geom *g, acts *a) {
  for (int v = 0; v < n->n_views; ++v)
    for (int l = 0; l <= n->n_conv; ++l)
      a->conv[v][l] = (double *)malloc(sizeof(double) * (size_t)g->c[l] * g->h[l] * g->w[l]);
  for (int l = 0; l <= n->n_conv; ++l)
    a->dconv[l] = (double *)malloc(sizeof(double) * (size_t)g->c[l] * g->h[l] * g->w[l]);
  a->feat = (double *)malloc(sizeof(double) * (size_t)g->feat);
  a->dfeat = (double *)malloc(sizeof(double) * (size_t)g->feat);
  for (int l = 0; l < n->n_fc; ++l) {
    a->fc[l] = (double *)malloc(sizeof(double) * (size_t)g->fc_out[l]);
    a->dfc[l] = (double *)malloc(sizeof(double) * (size_t)g->fc_out[l]);
  }
  a->mu = (double *)malloc(sizeof(double) * (size_t)n->act_dim);
}
static void acts_free(const orc_net *n, acts *a) {
  for (int v = 0; v < n->n_views; ++v)
    for (int l = 0; l <= n->n_conv; ++l) free(a->conv[v][l]);
  for (int l = 0; l <= n->n_conv; ++l) free(a->dconv[l]);
  free(a->feat); free(a->dfeat);
  for (int l = 0; l < n->n_fc; ++l) { free(a->fc[l]); free(a->dfc[l]); }
  free(a->mu);
}

/* Forward of one sample: conv stack (+bias, ReLU) on each view with shared
 * weights, flatten in (c,h,w) order, views side by side, append proprio,
 * hidden layers (+bias, ReLU), linear heads (no squashing). */
static void sample_forward(const orc_net *n, const geom *g, const double *P, const float *obs,
                           const double *proprio, acts *a) {
  for (int v = 0; v < n->n_views; ++v) {
    int64_t px = (int64_t)g->c[0] * g->h[0] * g->w[0];
    for (int64_t i = 0; i < px; ++i) a->conv[v][0][i] = q((double)obs[v * px + i]);  /* the stored image */
    for (int l = 0; l < n->n_conv; ++l) {
      conv_fwd(a->conv[v][l], g->c[l], g->h[l], g->w[l], P + g->convW[l], P + g->convB[l],
               g->c[l + 1], n->conv_k, n->conv_stride, n->conv_pad, a->conv[v][l + 1], g->h[l + 1],
               g->w[l + 1]);
      int64_t m = (int64_t)g->c[l + 1] * g->h[l + 1] * g->w[l + 1];
      for (int64_t i = 0; i < m; ++i)
        a->conv[v][l + 1][i] = (a->conv[v][l + 1][i] > 0.0) ? q(a->conv[v][l + 1][i]) : 0.0;
    }
    memcpy(a->feat + (size_t)v * g->flat, a->conv[v][n->n_conv], sizeof(double) * (size_t)g->flat);
  }
  for (int i = 0; i < n->proprio_dim; ++i) a->feat[n->n_views * g->flat + i] = q(proprio[i]);
  const double *x = a->feat;
  for (int l = 0; l < n->n_fc; ++l) {
    lin_fwd(x, g->fc_in[l], P + g->fcW[l], P + g->fcB[l], g->fc_out[l], a->fc[l]);
    for (int i = 0; i < g->fc_out[l]; ++i) a->fc[l][i] = (a->fc[l][i] > 0.0) ? q(a->fc[l][i]) : 0.0;
    x = a->fc[l];
  }
  lin_fwd(x, g->hid, P + g->muW, P + g->muB, n->act_dim, a->mu);
  a->v = 0.0;
  if (n->has_value_head) lin_fwd(x, g->hid, P + g->vW, P + g->vB, 1, &a->v);
}

/* Backward of one sample from dmu[A], dv; accumulates into G (param layout).
 * ReLU passes gradient where the stored activation is > 0. */
static void sample_backward(const orc_net *n, const geom *g, const double *P, acts *a,
                            const double *dmu, double dv, double *G) {
  const double *x = n->n_fc ? a->fc[n->n_fc - 1] : a->feat;
  double *dx = n->n_fc ? a->dfc[n->n_fc - 1] : a->dfeat;
  memset(dx, 0, sizeof(double) * (size_t)g->hid);
  lin_bwd(x, g->hid, P + g->muW, n->act_dim, dmu, G + g->muW, G + g->muB, dx);
  if (n->has_value_head) lin_bwd(x, g->hid, P + g->vW, 1, &dv, G + g->vW, G + g->vB, dx);
  for (int l = n->n_fc - 1; l >= 0; --l) {
    double *dy = a->dfc[l];
    for (int i = 0; i < g->fc_out[l]; ++i) dy[i] = (a->fc[l][i] > 0.0) ? q(dy[i]) : 0.0;
    const double *xin = l ? a->fc[l - 1] : a->feat;
    double *dxin = l ? a->dfc[l - 1] : a->dfeat;
    memset(dxin, 0, sizeof(double) * (size_t)g->fc_in[l]);
    lin_bwd(xin, g->fc_in[l], P + g->fcW[l], g->fc_out[l], dy, G + g->fcW[l], G + g->fcB[l], dxin);
  }
  for (int v = 0; v < n->n_views; ++v) {
    int L = n->n_conv;
    memcpy(a->dconv[L], a->dfeat + (size_t)v * g->flat, sizeof(double) * (size_t)g->flat);
    for (int l = L - 1; l >= 0; --l) {
      int64_t m = (int64_t)g->c[l + 1] * g->h[l + 1] * g->w[l + 1];
      for (int64_t i = 0; i < m; ++i)
        a->dconv[l + 1][i] = (a->conv[v][l + 1][i] > 0.0) ? q(a->dconv[l + 1][i]) : 0.0;
      double *dxl = l ? a->dconv[l] : NULL;
      if (dxl) memset(dxl, 0, sizeof(double) * (size_t)g->c[l] * g->h[l] * g->w[l]);
      conv_bwd(a->conv[v][l], g->c[l], g->h[l], g->w[l], P + g->convW[l], g->c[l + 1], n->conv_k,
               n->conv_stride, n->conv_pad, a->dconv[l + 1], g->h[l + 1], g->w[l + 1],
               G + g->convW[l], G + g->convB[l], dxl);
    }
  }
}

/* Copy of the parameters as the layers use them: in bf16-operand mode the weight matrices of
 * every layer are rounded to bf16; everything else is unchanged. */
static double *operand_params(const orc_net *n, const geom *g, const double *params) {
  double *P = (double *)malloc(sizeof(double) * (size_t)g->total);
  memcpy(P, params, sizeof(double) * (size_t)g->total);
  if (!g_quant) return P;
  for (int l = 0; l < n->n_conv; ++l)
    for (int64_t i = g->convW[l]; i < g->convB[l]; ++i) P[i] = q(P[i]);
  for (int l = 0; l < n->n_fc; ++l)
    for (int64_t i = g->fcW[l]; i < g->fcB[l]; ++i) P[i] = q(P[i]);
  for (int64_t i = g->muW; i < g->muB; ++i) P[i] = q(P[i]);
  if (n->has_value_head)
    for (int64_t i = g->vW; i < g->vB; ++i) P[i] = q(P[i]);
  return P;
}

/* Network outputs for B samples: mu [B][A], v [B] (v untouched without a value head). */
void orc_forward(const orc_net *n, const double *params_in, int64_t B, const float *obs,
                 const double *proprio, double *mu, double *v) {
  geom g; make_geom(n, &g);
  double *params = operand_params(n, &g, params_in);
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
#pragma omp parallel
  {
    acts a; acts_alloc(n, &g, &a);
#pragma omp for schedule(static)
    for (int64_t s = 0; s < B; ++s) {
      sample_forward(n, &g, params, obs + s * obs_sz, proprio + s * n->proprio_dim, &a);
      memcpy(mu + s * n->act_dim, a.mu, sizeof(double) * (size_t)n->act_dim);
      if (n->has_value_head) v[s] = a.v;
    }
    acts_free(n, &a);
  }
  free(params);
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

/* forward all samples, evaluate loss on the outputs, backward all samples */
static void minibatch_grad(const orc_net *n, const double *params_in, int64_t B, const float *obs,
                           const double *proprio, const double *action, const double *logp_old,
                           const double *v_old, const double *adv, const double *ret,
                           const orc_loss_cfg *cfg, int distill, double *grads, double *stats) {
  geom g; make_geom(n, &g);
  int A = n->act_dim;
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
  double *mu = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *v = (double *)calloc((size_t)B, sizeof(double));
  double *dmu = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *dv = (double *)calloc((size_t)B, sizeof(double));
  double *params = operand_params(n, &g, params_in);
  orc_forward(n, params_in, B, obs, proprio, mu, v);
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
    acts a; acts_alloc(n, &g, &a);
    double *G = tg + (size_t)tid * (size_t)g.total;
#pragma omp for schedule(static)
    for (int64_t s = 0; s < B; ++s) {
      sample_forward(n, &g, params, obs + s * obs_sz, proprio + s * n->proprio_dim, &a);
      sample_backward(n, &g, params, &a, dmu + s * A, dv[s], G);
    }
    acts_free(n, &a);
  }
  for (int t = 0; t < nth; ++t)
    for (int64_t i = 0; i < g.total; ++i) grads[i] += tg[(size_t)t * (size_t)g.total + i];
  double gn = 0;
  for (int64_t i = 0; i < g.total; ++i) gn += grads[i] * grads[i];
  stats[ST_GNORM] = sqrt(gn);
  free(tg); free(mu); free(v); free(dmu); free(dv); free(params);
}

/* Loss, stats and parameter gradients of the PPO objective on one minibatch. */
void orc_ppo_loss_grad(const orc_net *n, const double *params, int64_t B, const float *obs,
                       const double *proprio, const double *action, const double *logp_old,
                       const double *v_old, const double *adv, const double *ret,
                       const orc_loss_cfg *cfg, double *grads, double *stats) {
  minibatch_grad(n, params, B, obs, proprio, action, logp_old, v_old, adv, ret, cfg, 0, grads, stats);
}
void orc_distill_loss_grad(const orc_net *n, const double *params, int64_t B, const float *obs,
                           const double *proprio, const double *teacher, int32_t aux_dim,
                           double aux_coef, double *grads, double *stats) {
  orc_loss_cfg lc; memset(&lc, 0, sizeof lc); lc.aux_dim = aux_dim; lc.aux_coef = aux_coef;
  minibatch_grad(n, params, B, obs, proprio, teacher, NULL, NULL, NULL, NULL, &lc, 1, grads, stats);
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

/* One learner update over a buffer of S = N*T samples: for each epoch draw a
 * fresh permutation, split it into `minibatches` contiguous chunks, and for
 * each chunk: forward, loss, backward, one Adam step.  adv/ret/logp_old/v_old
 * stay fixed for the whole update.  *step is the Adam step counter (in/out).
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
                        int64_t S, const float *obs, const double *proprio, const double *action,
                        const double *logp_old, const double *v_old, const double *adv,
                        const double *ret, const orc_loss_cfg *lc, const orc_adam_cfg *ac,
                        int32_t epochs, int32_t minibatches, uint64_t seed, uint64_t update_idx,
                        int distill, double *stats, double *grads_last) {
  geom g; make_geom(n, &g);
  int A = n->act_dim, P = n->proprio_dim;
  int64_t obs_sz = (int64_t)n->n_views * g.c[0] * g.h[0] * g.w[0];
  int64_t B = S / minibatches;
  int32_t *perm = (int32_t *)malloc(sizeof(int32_t) * (size_t)S);
  float *mobs = (float *)malloc(sizeof(float) * (size_t)B * (size_t)obs_sz);
  double *mpro = (double *)malloc(sizeof(double) * (size_t)B * P);
  double *mact = (double *)malloc(sizeof(double) * (size_t)B * A);
  double *mlp = (double *)calloc((size_t)B, sizeof(double)), *mvo = (double *)calloc((size_t)B, sizeof(double));
  double *mad = (double *)calloc((size_t)B, sizeof(double)), *mre = (double *)calloc((size_t)B, sizeof(double));
  double *grads = (double *)malloc(sizeof(double) * (size_t)g.total);
  orc_adam_cfg cur = *ac;
  for (int e = 0; e < epochs; ++e) {
    orc_permutation(seed, update_idx, (uint64_t)e, S, perm);
    for (int mb = 0; mb < minibatches; ++mb) {
      for (int64_t b = 0; b < B; ++b) {
        int64_t s = perm[(int64_t)mb * B + b];
        memcpy(mobs + b * obs_sz, obs + s * obs_sz, sizeof(float) * (size_t)obs_sz);
        memcpy(mpro + b * P, proprio + s * P, sizeof(double) * (size_t)P);
        memcpy(mact + b * A, action + s * A, sizeof(double) * (size_t)A);
        if (!distill) { mlp[b] = logp_old[s]; mvo[b] = v_old[s]; mad[b] = adv[s]; mre[b] = ret[s]; }
      }
      double *st = stats + ((int64_t)e * minibatches + mb) * ST_N;
      minibatch_grad(n, params, B, mobs, mpro, mact, mlp, mvo, mad, mre, lc, distill, grads, st);
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
  free(perm); free(mobs); free(mpro); free(mact); free(mlp); free(mvo); free(mad); free(mre); free(grads);
}

void orc_ppo_update(const orc_net *n, double *params, double *m, double *v, int64_t *step, int64_t S,
                    const float *obs, const double *proprio, const double *action,
                    const double *logp_old, const double *v_old, const double *adv,
                    const double *ret, const orc_loss_cfg *lc, const orc_adam_cfg *ac,
                    int32_t epochs, int32_t minibatches, uint64_t seed, uint64_t update_idx,
                    double *stats, double *grads_last) {
  update_loop(n, params, m, v, step, S, obs, proprio, action, logp_old, v_old, adv, ret, lc, ac,
              epochs, minibatches, seed, update_idx, 0, stats, grads_last);
}
void orc_distill_update(const orc_net *n, double *params, double *m, double *v, int64_t *step,
                        int64_t S, const float *obs, const double *proprio, const double *teacher,
                        int32_t aux_dim, double aux_coef,
                        const orc_adam_cfg *ac, int32_t epochs, int32_t minibatches, uint64_t seed,
                        uint64_t update_idx, double *stats, double *grads_last) {
  orc_loss_cfg lc; memset(&lc, 0, sizeof lc); lc.aux_dim = aux_dim; lc.aux_coef = aux_coef;
  update_loop(n, params, m, v, step, S, obs, proprio, teacher, NULL, NULL, NULL, NULL, &lc, ac,
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
