// Host side of libppo_learner.so: context, argument validation, parameter layout, and the
// launch sequences of ppo_buffer_write / ppo_gae / ppo_update / distill_update.
// Every step of the learner's path runs in the HIP kernels of gemm.hip.h and mem_kernels.hip.h.
#include "../../include/ppo_learner.h"
#include "../../include/ppo_learner_diag.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <map>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "gemm.hip.h"
#include "gemm_dma.hip.h"
#include "mem_kernels.hip.h"
#include "fused.hip.h"
#include "conv_tile.hip.h"
#include "conv_dgrad_tile.hip.h"
#include "conv_dgrad_wgrad0_tile.hip.h"
#include "conv_dgrad_k2_tile.hip.h"
#include "conv0_tile.hip.h"
#include "head_loss.hip.h"
#include "wgrad_rs.hip.h"
#include "peaks.hip.h"
#include "recurrent.hip.h"

static_assert(sizeof(DevStats) == sizeof(ppo_mb_stats), "device and host statistics records must match");

// Scratch of ppo_permutation_static: bucket histogram + cursors [2*nb], bucket starts [nb], bucket-ordered
// indices [S], for up to STATIC_PERM_MAX_S samples (nb <= STATIC_PERM_MAX_NB buckets of about 32 keys).  Every GPU
// the library runs on holds its own copy of this array until the process ends (4.4 MiB).
constexpr int64_t STATIC_PERM_MAX_S = 1 << 20;
constexpr int STATIC_PERM_MAX_NB = 1 << 15;
constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) int32_t scratch[3 * STATIC_PERM_MAX_NB + STATIC_PERM_MAX_S];

namespace {

thread_local std::string g_create_error;

// Device address of `scratch` on the current device.  In host code the array's name is only a stand-in for the
// symbol, not an address a kernel can use: the address is asked for once per device (with that device current)
// and kept; host code passes this pointer, never the name, to kernels.
std::mutex g_scratch_mutex;
int32_t* g_scratch_ptr[STATIC_MAX_DEVICES] = {};
hipError_t static_scratch(int32_t** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = (int32_t*)p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

struct Ctx {
  ppo_net_desc d;
  hipStream_t stream = nullptr;
  int dev = 0;  // the HIP device the context lives on (kernel attributes are set once per device)
  std::string err;
  // geometry
  int N = 0, T = 0, S = 0, V = 1, A = 0, P = 0, NH = 0, nconv = 0, nfc = 0;
  int cC[PPO_MAX_LAYERS + 1], cH[PPO_MAX_LAYERS + 1], cW[PPO_MAX_LAYERS + 1];
  int fin[PPO_MAX_LAYERS], fout[PPO_MAX_LAYERS];
  int flat = 0, feat_ld = 0, hid = 0;
  int64_t img_elems = 0;  // per view
  // internal parameter layout (fp32 master, bf16 shadow share the offsets)
  int64_t convW[PPO_MAX_LAYERS], convB[PPO_MAX_LAYERS], fcW[PPO_MAX_LAYERS], fcB[PPO_MAX_LAYERS];
  int64_t headW = 0, headB = 0, logstd = -1, total = 0;
  // optional parts of the network
  int XH = 0, X = 0, A_main = 0;            // auxiliary MLP head: hidden width, outputs; rows of the linear mean head
  int64_t aux1W = -1, aux1B = -1, aux2W = -1, aux2B = -1;
  bool ln = false;                          // layer normalisation after every convolution
  int64_t lnG[PPO_MAX_LAYERS], lnB[PPO_MAX_LAYERS];
  int E = 0, enc = 0;                       // embedding width (0: none); encoder output width per view
  int64_t embW = -1, embB = -1;
  int nl = 0, H = 0, lin[4] = {0, 0, 0, 0};  // LSTM layers, units, input width per layer
  int64_t lstmW[4], lstmB[4];               // per layer [4H][lin + H] (input and recurrent weights side by side), bias [4H]
  int feat_cols = 0;                        // V*enc + P: the feature columns of a row of the feature matrix
  // workspaces of the generic encoder (layer norm and / or embedding) and of the recurrent core
  bf16_t* pre[PPO_MAX_LAYERS] = {};         // conv outputs before the layer normalisation [CH*V][Ho*Wo*Co]
  float2* lnstat[PPO_MAX_LAYERS] = {};      // (mean, rstd) per image
  bf16_t* dpre = nullptr;                   // gradient w.r.t. one convolution's output (largest layer)
  bf16_t* embT = nullptr;                   // [flat][E]
  bf16_t* lstmWT[4] = {};                   // [lin + H][4H]
  bf16_t* xh[4] = {};                       // LSTM layer inputs [CH][lin + H]: x_t, then the h entering step t (xh[0] is the feature matrix)
  bf16_t* dxh[4] = {};                      // their gradients
  float* gates[4] = {};                     // [CH][4H] gate activations
  float* c_enter[4] = {};                   // [CH][H] cell state entering each step
  float* lstm_pre = nullptr;                // [CHe][4H] gate pre-activations of one step
  bf16_t* da = nullptr;                     // [CH][4H] gate pre-activation gradients of one layer
  float* dc_carry = nullptr;                // [CHe][H]
  bf16_t* htop = nullptr;                   // [CH][H] top layer's h: the trunk's input
  int32_t* seqidx = nullptr;                // [CH] rollout sample of each row of a sequence chunk
  float *h0 = nullptr, *c0 = nullptr;       // [nl][N][H] state of every environment at the start of the rollout
  int PU = 0;                               // units the minibatch permutation shuffles: N environments (recurrent) or S samples
  int CHe = 0;                              // environments per sequence chunk
  std::vector<int32_t> i2c;  // internal index -> canonical index
  // device: parameters
  float *p = nullptr, *m = nullptr, *v = nullptr, *g = nullptr;
  bf16_t* shadow = nullptr;
  bf16_t* wd[PPO_MAX_LAYERS][2];  // transposed-conv weights per row parity (conv layers >= 1)
  bf16_t* wtap[PPO_MAX_LAYERS];   // the same weights transposed per tap: [9][Cin][Cout]
  uint32_t* abits[PPO_MAX_LAYERS] = {};  // sign bits of conv layer l's stored output for the current chunk (ReLU mask of the backward pass)
  bool abits_ok[PPO_MAX_LAYERS] = {};    // written by the forward kernel that ran for this chunk
  int64_t wver = 0;                      // bumped whenever the weights change (every repack_weights call)
  int64_t wd_ver[PPO_MAX_LAYERS] = {};   // weight version that wd[l] holds (0: none); packed on demand
  bf16_t* fcT[PPO_MAX_LAYERS];    // [in][out]
  bf16_t* headT = nullptr;        // [hid][32]
  bf16_t *aux1T = nullptr, *aux2T = nullptr;  // auxiliary head: [hid][XH], [XH][32]
  bf16_t *auxact = nullptr, *dauxact = nullptr, *daux = nullptr;  // its hidden activation [CH][XH], that layer's gradient, its output gradient [CH][32]
  // device: rollout buffer (SoA)
  bf16_t *obs = nullptr, *proprio = nullptr;
  float *action = nullptr, *logp = nullptr, *value = nullptr, *reward = nullptr, *adv = nullptr, *ret = nullptr;
  uint8_t* done = nullptr;
  // device: permutation
  int32_t *perm = nullptr, *ptmp = nullptr, *phist = nullptr, *pstart = nullptr;
  int nb = 1, shift = 64;
  // device: workspaces for one chunk of CH samples
  int CH = 0;
  bf16_t* act[PPO_MAX_LAYERS];    // conv outputs of layers 0..nconv-2, [CH*V][H][W][C]
  bf16_t* feat = nullptr;         // [CH][feat_ld]: last conv output per view, then proprio
  bf16_t* fcact[PPO_MAX_LAYERS];  // [CH][fout]
  float* headout = nullptr;       // [CH][32]
  bf16_t* dhead = nullptr;        // [CH][32]
  bf16_t* gbuf[2] = {nullptr, nullptr};
  float *partial = nullptr, *bias_partial = nullptr;
  bf16_t* zpage = nullptr;  // 64 KiB of zeros: source of out-of-range operand fetches (most kernels use its first KiB)
  // partial / bias_partial are cursors into the two workspaces and *_elems what is left behind them:
  // every weight-gradient kernel of a backward pass takes its partials from the cursor and queues its
  // reduction (defer_reduce); flush_reduces sums them all in one launch and rewinds the cursors
  int64_t partial_elems = 0, bias_partial_elems = 0;
  float *partial_base = nullptr, *bias_partial_base = nullptr;
  int64_t partial_cap = 0, bias_partial_cap = 0;
  ReduceJobs rjobs;
  LossFinalize lossfin = {};    // pending: rides as the last block of the next reduction launch
  GnormFinalize gnfin = {}; // pending: rides as the last block of the next re-pack launch
  int rjob_blocks = 0;
  float *stat_part = nullptr, *dls_part = nullptr, *sq_part = nullptr, *clip_coef = nullptr;
  float* lr_dev = nullptr;  // the KL-adaptive learning rate (desired_kl > 0); lr_live: an adaptive update has left a rate there
  bool lr_live = false;
  float* adv_n = nullptr;  // advantages normalised over the rollout (norm_adv)
  float* advn_part = nullptr;  // per-block (count, mean, squared deviations) of that normalisation
  int max_loss_blocks = 0, adam_blocks = 0;
  DevStats* dstats = nullptr;
  int max_steps = 4096;
  // state
  std::vector<char> written;                               // per step: 0 incomplete, 1 complete, 2 acted (outcome missing)
  std::vector<std::vector<std::pair<int, int>>> cover;     // per step: merged environment ranges of partial writes
  bool gae_done = false;
  int64_t step = 0, update_idx = 0;
  std::vector<void*> allocs;
  // optional per-kernel-class timing with HIP events on the context's stream
  bool prof_on = false;
  struct ProfClass { std::string name; int64_t launches = 0; double flops = 0, bytes = 0; };
  struct ProfRec { int cls; hipEvent_t a, b; };
  std::vector<ProfClass> prof_cls;
  std::map<std::string, int> prof_idx;
  std::vector<ProfRec> prof_recs;
  std::vector<hipEvent_t> prof_pool;
};

// Brackets the launches made during its lifetime with a pair of events (when profiling is on) and
// books the algorithmic FLOPs / bytes of the work under `name`.
struct ProfScope {
  Ctx* c; int rec = -1;
  ProfScope(Ctx* c_, const std::string& name, double flops, double bytes) : c(c_) {
    if (!c->prof_on) return;
    auto it = c->prof_idx.find(name);
    int id;
    if (it == c->prof_idx.end()) { id = (int)c->prof_cls.size(); c->prof_idx[name] = id; Ctx::ProfClass pc; pc.name = name; c->prof_cls.push_back(pc); }
    else id = it->second;
    c->prof_cls[id].launches += 1; c->prof_cls[id].flops += flops; c->prof_cls[id].bytes += bytes;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!c->prof_pool.empty()) { ev[i] = c->prof_pool.back(); c->prof_pool.pop_back(); }
      else if (hipEventCreate(&ev[i]) != hipSuccess) return;
    }
    Ctx::ProfRec r; r.cls = id; r.a = ev[0]; r.b = ev[1];
    (void)hipEventRecord(r.a, c->stream);
    rec = (int)c->prof_recs.size();
    c->prof_recs.push_back(r);
  }
  ~ProfScope() { if (rec >= 0) (void)hipEventRecord(c->prof_recs[rec].b, c->stream); }
};

int fail(Ctx* c, int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_create_error = buf;
  return code;
}

#define HIPCHK(c, call)                                                                          \
  do {                                                                                           \
    hipError_t e_ = (call);                                                                      \
    if (e_ != hipSuccess) return fail(c, PPO_EHIP, "%s failed: %s", #call, hipGetErrorString(e_)); \
  } while (0)
#define LAUNCHCHK(c, what)                                                                              \
  do {                                                                                                  \
    hipError_t e_ = hipGetLastError();                                                                  \
    if (e_ != hipSuccess) return fail(c, PPO_EHIP, "launch of %s failed: %s", what, hipGetErrorString(e_)); \
  } while (0)

template <typename T>
int dalloc(Ctx* c, T** out, int64_t n) {
  void* p = nullptr;
  size_t bytes = (size_t)(n > 0 ? n : 1) * sizeof(T);
  hipError_t e = hipMalloc(&p, bytes);
  if (e != hipSuccess) return fail(c, e == hipErrorOutOfMemory ? PPO_ENOMEM : PPO_EHIP, "hipMalloc of %zu bytes failed: %s", bytes, hipGetErrorString(e));
  c->allocs.push_back(p);
  *out = (T*)p;
  return PPO_OK;
}
#define DALLOC(c, ptr, n)                          \
  do {                                             \
    int rc_ = dalloc(c, &(ptr), (int64_t)(n));     \
    if (rc_ != PPO_OK) return rc_;                 \
  } while (0)

inline int cdiv(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// ---------------------------------------------------------------- validation (no HIP calls)
int validate_desc(const ppo_net_desc* d) {
  if (!d) return fail(nullptr, PPO_EINVAL, "desc is NULL");
  if (d->num_envs < 1 || d->horizon < 1) return fail(nullptr, PPO_ESHAPE, "num_envs and horizon must be >= 1");
  if ((int64_t)d->num_envs * d->horizon > (1 << 30)) return fail(nullptr, PPO_ESHAPE, "num_envs*horizon too large");
  if (d->n_views < 1 || d->n_views > 4) return fail(nullptr, PPO_ESHAPE, "n_views must be 1..4");
  if (d->in_c != 1 && d->in_c != 3) return fail(nullptr, PPO_ESHAPE, "in_c must be 1 (depth) or 3 (RGB)");
  if (d->in_h < 2 || d->in_w < 2 || d->in_h > 4096 || d->in_w > 4096) return fail(nullptr, PPO_ESHAPE, "image size out of range");
  if (d->obs_dtype != 0 && d->obs_dtype != 1) return fail(nullptr, PPO_EINVAL, "obs_dtype must be 0 (fp32) or 1 (bf16)");
  if (d->proprio_dim < 8 || d->proprio_dim % 8) return fail(nullptr, PPO_ESHAPE, "proprio_dim must be a positive multiple of 8");
  if (d->act_dim < 1 || d->act_dim > 31) return fail(nullptr, PPO_ESHAPE, "act_dim must be 1..31");
  if (d->conv_k != 3 || d->conv_stride != 2 || d->conv_pad != 1) return fail(nullptr, PPO_ESHAPE, "only 3x3 stride-2 pad-1 convolutions are supported");
  if (d->n_conv < 2 || d->n_conv > PPO_MAX_LAYERS) return fail(nullptr, PPO_ESHAPE, "n_conv must be 2..%d", PPO_MAX_LAYERS);
  for (int i = 0; i < d->n_conv; ++i)
    if (d->conv_ch[i] < 8 || d->conv_ch[i] > 1024 || (d->conv_ch[i] & (d->conv_ch[i] - 1))) return fail(nullptr, PPO_ESHAPE, "conv_ch[%d] must be a power of two in 8..1024", i);
  if (d->conv_ch[0] != 8 && d->conv_ch[0] != 16 && d->conv_ch[0] != 32 && d->conv_ch[0] != 64) return fail(nullptr, PPO_ESHAPE, "conv_ch[0] must be 8, 16, 32 or 64");
  if (d->n_fc < 1 || d->n_fc > PPO_MAX_LAYERS) return fail(nullptr, PPO_ESHAPE, "n_fc must be 1..%d", PPO_MAX_LAYERS);
  for (int i = 0; i < d->n_fc; ++i)
    if (d->fc_dim[i] < 8 || d->fc_dim[i] % 8 || d->fc_dim[i] > 16384) return fail(nullptr, PPO_ESHAPE, "fc_dim[%d] must be a multiple of 8 in 8..16384", i);
  if (d->has_value_head != 0 && d->has_value_head != 1) return fail(nullptr, PPO_EINVAL, "has_value_head must be 0 or 1");
  if (d->max_chunk < 0) return fail(nullptr, PPO_EINVAL, "max_chunk must be >= 0");
  if (d->aux_hidden < 0 || d->aux_hidden % 8 || d->aux_hidden > 4096) return fail(nullptr, PPO_ESHAPE, "aux_hidden must be a multiple of 8 in 0..4096");
  if (d->aux_hidden > 0 && d->has_value_head) return fail(nullptr, PPO_ESHAPE, "the auxiliary MLP head belongs to a distillation student (has_value_head = 0)");
  if (d->aux_hidden > 0 && (d->aux_dim < 1 || d->aux_dim >= d->act_dim)) return fail(nullptr, PPO_ESHAPE, "aux_dim must be in 1..act_dim-1 when aux_hidden > 0");
  if (d->aux_hidden == 0 && d->aux_dim != 0) return fail(nullptr, PPO_ESHAPE, "aux_dim without aux_hidden (for auxiliary columns of the linear head use ppo_hparams.aux_dim)");
  if (d->layer_norm != 0 && d->layer_norm != 1) return fail(nullptr, PPO_EINVAL, "layer_norm must be 0 or 1");
  if (d->embed_dim < 0 || d->embed_dim % 8 || d->embed_dim > 4096) return fail(nullptr, PPO_ESHAPE, "embed_dim must be a multiple of 8 in 0..4096");
  if (d->lstm_layers < 0 || d->lstm_layers > 4) return fail(nullptr, PPO_ESHAPE, "lstm_layers must be 0..4");
  if (d->lstm_layers > 0 && (d->lstm_units < 8 || d->lstm_units % 8 || d->lstm_units > 4096)) return fail(nullptr, PPO_ESHAPE, "lstm_units must be a multiple of 8 in 8..4096");
  if (d->lstm_layers == 0 && d->lstm_units != 0) return fail(nullptr, PPO_ESHAPE, "lstm_units without lstm_layers");
  if (d->lstm_layers > 0 && !d->has_value_head) return fail(nullptr, PPO_ESHAPE, "recurrent layers are built for the actor-critic teacher (has_value_head = 1)");
  return PPO_OK;
}

int validate_hp(Ctx* c, const ppo_hparams* hp, bool distill) {
  if (!hp) return fail(c, PPO_EINVAL, "hparams is NULL");
  const float f[] = {hp->clip_eps, hp->vclip_eps, hp->vf_coef, hp->ent_coef, hp->lr, hp->beta1, hp->beta2, hp->adam_eps, hp->max_grad_norm, hp->desired_kl, hp->aux_coef};
  for (float x : f) if (!isfinite(x)) return fail(c, PPO_EINVAL, "non-finite hyper-parameter");
  if (!distill && !(hp->clip_eps > 0.f)) return fail(c, PPO_EINVAL, "clip_eps must be > 0");
  if (!(hp->lr >= 0.f) || !(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f) || !(hp->adam_eps > 0.f))
    return fail(c, PPO_EINVAL, "Adam hyper-parameters out of range");
  if (hp->norm_adv != 0 && hp->norm_adv != 1) return fail(c, PPO_EINVAL, "norm_adv must be 0 or 1");
  if (hp->lr_carry != 0 && hp->lr_carry != 1) return fail(c, PPO_EINVAL, "lr_carry must be 0 or 1");
  if (distill && (hp->aux_dim < 0 || hp->aux_dim >= c->A)) return fail(c, PPO_EINVAL, "aux_dim must be in [0, act_dim)");
  if (distill && hp->aux_dim > 0 && !(hp->aux_coef >= 0.f)) return fail(c, PPO_EINVAL, "aux_coef must be >= 0");
  if (distill && c->XH > 0 && hp->aux_dim != c->X) return fail(c, PPO_EINVAL, "this student has an auxiliary MLP head for %d outputs: hparams.aux_dim must be %d", c->X, c->X);
  if (!distill && hp->desired_kl > 0.f && !(isfinite(hp->lr_min) && isfinite(hp->lr_max) && hp->lr_min > 0.f && hp->lr_min <= hp->lr_max))
    return fail(c, PPO_EINVAL, "desired_kl > 0 needs 0 < lr_min <= lr_max");
  if (hp->epochs < 1 || hp->minibatches < 1) return fail(c, PPO_EINVAL, "epochs and minibatches must be >= 1");
  if (c->PU % hp->minibatches)
    return fail(c, PPO_ESHAPE, "%s = %d is not divisible by minibatches = %d", c->nl > 0 ? "num_envs (a recurrent net's minibatches are whole environments)" : "num_envs*horizon",
                c->PU, hp->minibatches);
  if ((int64_t)hp->epochs * hp->minibatches > c->max_steps) return fail(c, PPO_ESHAPE, "epochs*minibatches exceeds %d", c->max_steps);
  return PPO_OK;
}

// ---------------------------------------------------------------- geometry and parameter layout
void build_geometry(Ctx* c) {
  const ppo_net_desc& d = c->d;
  c->N = d.num_envs; c->T = d.horizon; c->S = c->N * c->T; c->V = d.n_views; c->A = d.act_dim; c->P = d.proprio_dim;
  c->XH = d.aux_hidden; c->X = d.aux_hidden > 0 ? d.aux_dim : 0; c->A_main = c->A - c->X;
  c->ln = d.layer_norm != 0; c->E = d.embed_dim; c->nl = d.lstm_layers; c->H = d.lstm_layers > 0 ? d.lstm_units : 0;
  c->NH = c->A_main + (d.has_value_head ? 1 : 0);
  c->nconv = d.n_conv; c->nfc = d.n_fc;
  c->cC[0] = d.in_c; c->cH[0] = d.in_h; c->cW[0] = d.in_w;
  for (int l = 0; l < c->nconv; ++l) {
    c->cC[l + 1] = d.conv_ch[l];
    c->cH[l + 1] = (c->cH[l] + 2 - 3) / 2 + 1;
    c->cW[l + 1] = (c->cW[l] + 2 - 3) / 2 + 1;
  }
  c->img_elems = (int64_t)d.in_c * d.in_h * d.in_w;
  c->flat = c->cC[c->nconv] * c->cH[c->nconv] * c->cW[c->nconv];
  c->enc = c->E > 0 ? c->E : c->flat;
  c->feat_cols = c->V * c->enc + c->P;
  // recurrent nets: a feature row is followed by the h that enters the first LSTM layer at that step (the two
  // halves of that layer's GEMM operand side by side)
  c->feat_ld = c->feat_cols + (c->nl > 0 ? c->H : 0);
  int in = c->feat_cols;
  for (int l = 0; l < c->nl; ++l) { c->lin[l] = in; in = c->H; }
  for (int l = 0; l < c->nfc; ++l) { c->fin[l] = in; c->fout[l] = d.fc_dim[l]; in = d.fc_dim[l]; }
  c->hid = in;

  // canonical offsets: per conv W, b, [gain, shift]; [embedding W, b]; per LSTM layer W_ih, W_hh, b; per hidden
  // layer W, b; mean head W, b; [value head w, b; logstd]; [auxiliary head W1, b1, W2, b2]
  std::vector<int64_t> cConvW(c->nconv), cConvB(c->nconv), cLnG(c->nconv), cLnB(c->nconv), cFcW(c->nfc), cFcB(c->nfc);
  int64_t cWih[4], cWhh[4], cLb[4], cEmbW = -1, cEmbB = -1;
  int64_t off = 0;
  for (int l = 0; l < c->nconv; ++l) {
    cConvW[l] = off; off += (int64_t)c->cC[l + 1] * c->cC[l] * 9; cConvB[l] = off; off += c->cC[l + 1];
    if (c->ln) { cLnG[l] = off; off += c->cC[l + 1]; cLnB[l] = off; off += c->cC[l + 1]; }
  }
  if (c->E > 0) { cEmbW = off; off += (int64_t)c->E * c->flat; cEmbB = off; off += c->E; }
  for (int l = 0; l < c->nl; ++l) {
    cWih[l] = off; off += (int64_t)4 * c->H * c->lin[l]; cWhh[l] = off; off += (int64_t)4 * c->H * c->H; cLb[l] = off; off += 4 * c->H;
  }
  for (int l = 0; l < c->nfc; ++l) { cFcW[l] = off; off += (int64_t)c->fin[l] * c->fout[l]; cFcB[l] = off; off += c->fout[l]; }
  int64_t cMuW = off; off += (int64_t)c->A_main * c->hid;
  int64_t cMuB = off; off += c->A_main;
  int64_t cVW = -1, cVB = -1, cLs = -1;
  if (d.has_value_head) { cVW = off; off += c->hid; cVB = off; off += 1; cLs = off; off += c->A; }
  int64_t cA1W = -1, cA1B = -1, cA2W = -1, cA2B = -1;
  if (c->XH > 0) {
    cA1W = off; off += (int64_t)c->XH * c->hid; cA1B = off; off += c->XH;
    cA2W = off; off += (int64_t)c->X * c->XH; cA2B = off; off += c->X;
  }
  c->total = off;
  c->i2c.assign((size_t)off, 0);
  auto same = [&](int64_t io, int64_t co, int64_t n) { for (int64_t i = 0; i < n; ++i) c->i2c[(size_t)(io + i)] = (int32_t)(co + i); };

  // internal layout: conv W as [Co][(u*3+v)*Ci + ci]; the first layer behind the convolutions reads the
  // channel-last flatten (view, pixel, channel); LSTM input and recurrent weights side by side per gate row;
  // heads stacked as one [NH][hid] matrix.  Every matrix starts at a multiple of 8 elements (16-byte operand
  // loads from the bf16 shadow) and every bias a bf16-output epilogue reads at a multiple of 4: the vectors of
  // odd length (head biases, log-std, the auxiliary output bias) come last.
  int64_t io = 0;
  for (int l = 0; l < c->nconv; ++l) {
    int Co = c->cC[l + 1], Ci = c->cC[l];
    c->convW[l] = io;
    for (int co = 0; co < Co; ++co)
      for (int u = 0; u < 3; ++u)
        for (int v = 0; v < 3; ++v)
          for (int ci = 0; ci < Ci; ++ci)
            c->i2c[(size_t)(io + (int64_t)co * 9 * Ci + (u * 3 + v) * Ci + ci)] = (int32_t)(cConvW[l] + (((int64_t)co * Ci + ci) * 3 + u) * 3 + v);
    io += (int64_t)Co * 9 * Ci;
    c->convB[l] = io; same(io, cConvB[l], Co); io += Co;
    c->lnG[l] = c->lnB[l] = -1;
    if (c->ln) { c->lnG[l] = io; same(io, cLnG[l], Co); io += Co; c->lnB[l] = io; same(io, cLnB[l], Co); io += Co; }
  }
  const int CL = c->cC[c->nconv], HWL = c->cH[c->nconv] * c->cW[c->nconv];
  // column j of a matrix that reads the channel-last flatten of one view <-> canonical (c,h,w) column
  auto flat_col = [&](int r) { const int pix = r / CL, ch = r - pix * CL; return ch * HWL + pix; };
  if (c->E > 0) {
    c->embW = io;
    for (int o = 0; o < c->E; ++o)
      for (int j = 0; j < c->flat; ++j) c->i2c[(size_t)(io + (int64_t)o * c->flat + j)] = (int32_t)(cEmbW + (int64_t)o * c->flat + flat_col(j));
    io += (int64_t)c->E * c->flat;
    c->embB = io; same(io, cEmbB, c->E); io += c->E;
  }
  // the first layer behind the concatenation [encoder(view 0), ..., proprioception]
  auto feat_col = [&](int j) {
    if (c->E > 0 || j >= c->V * c->flat) return j;
    const int v = j / c->flat;
    return v * c->flat + flat_col(j - v * c->flat);
  };
  for (int l = 0; l < c->nl; ++l) {
    const int K = c->lin[l] + c->H;
    c->lstmW[l] = io;
    for (int r = 0; r < 4 * c->H; ++r) {
      for (int j = 0; j < c->lin[l]; ++j)
        c->i2c[(size_t)(io + (int64_t)r * K + j)] = (int32_t)(cWih[l] + (int64_t)r * c->lin[l] + (l == 0 ? feat_col(j) : j));
      for (int j = 0; j < c->H; ++j) c->i2c[(size_t)(io + (int64_t)r * K + c->lin[l] + j)] = (int32_t)(cWhh[l] + (int64_t)r * c->H + j);
    }
    io += (int64_t)4 * c->H * K;
    c->lstmB[l] = io; same(io, cLb[l], 4 * c->H); io += 4 * c->H;
  }
  for (int l = 0; l < c->nfc; ++l) {
    c->fcW[l] = io;
    for (int o = 0; o < c->fout[l]; ++o)
      for (int j = 0; j < c->fin[l]; ++j)
        c->i2c[(size_t)(io + (int64_t)o * c->fin[l] + j)] = (int32_t)(cFcW[l] + (int64_t)o * c->fin[l] + ((l == 0 && c->nl == 0) ? feat_col(j) : j));
    io += (int64_t)c->fin[l] * c->fout[l];
    c->fcB[l] = io; same(io, cFcB[l], c->fout[l]); io += c->fout[l];
  }
  if (c->XH > 0) {
    c->aux1W = io; same(io, cA1W, (int64_t)c->XH * c->hid); io += (int64_t)c->XH * c->hid;
    c->aux1B = io; same(io, cA1B, c->XH); io += c->XH;
    c->aux2W = io; same(io, cA2W, (int64_t)c->X * c->XH); io += (int64_t)c->X * c->XH;
  }
  c->headW = io; same(io, cMuW, (int64_t)c->A_main * c->hid); io += (int64_t)c->A_main * c->hid;
  if (d.has_value_head) { same(io, cVW, c->hid); io += c->hid; }
  c->headB = io; same(io, cMuB, c->A_main); io += c->A_main;
  if (d.has_value_head) {
    c->i2c[(size_t)io] = (int32_t)cVB; io += 1;
    c->logstd = io; same(io, cLs, c->A); io += c->A;
  }
  if (c->XH > 0) { c->aux2B = io; same(io, cA2B, c->X); io += c->X; }
}

// number of input pixels of parity `par` along an axis of length n
inline int class_len(int n, int par) { return (n - par + 1) / 2; }

// ---------------------------------------------------------------- launch helpers
inline int ilog2(int x) { int l = 0; while ((1 << l) < x) ++l; return l; }

template <class AL, class EP>
int launch_gemm(Ctx* c, const AL& al_, int M, const bf16_t* Bm, int64_t ldb, int N, int K, const EP& ep_, const std::string& name, double abytes,
                int zdim = 1, double flops = -1.0) {
  if (M <= 0) return PPO_OK;
  AL al = al_; EP ep = ep_;
  al.prepare(); ep.map.prepare();
  const char* what = name.c_str();
  ProfScope ps(c, name, flops >= 0.0 ? flops : 2.0 * M * (double)N * K, abytes);
  dim3 blk(256);
  // Very deep reductions stream their operands through an LDS ring of up to eight stages, filled by
  // four loader waves while four or eight other waves compute (k_gemm_rs); medium ones take 64-wide
  // steps through registers, where the smaller LDS footprint lets more blocks share a CU and hide
  // the prologue and epilogue of their short loops.
#define LAUNCH_GEMM_RS(BM_, BN_, WM_, WN_)                                                                              \
  do {                                                                                                                   \
    constexpr int ncw = WM_ * WN_;                                                                                       \
    constexpr int nst = (BM_ + BN_) * 128 * 8 <= 128 * 1024 ? 8 : ((BM_ + BN_) * 128 * 4 <= 128 * 1024 ? 4 : 3);            \
    auto kfn = k_gemm_rs<BM_, BN_, WM_, WN_, nst, AL, EP>;                                                               \
    constexpr int lds = nst * (BM_ + BN_) * 128;                                                                         \
    static uint64_t attr_devs = 0;  /* bit d: set on device d */                                                                                        \
    if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, lds)); attr_devs |= 1ull << c->dev; } \
    hipLaunchKernelGGL(kfn, grid, dim3((ncw + 4) * 64), lds, c->stream, al, Bm, ldb, N, ep, c->zpage);                    \
  } while (0)
#define LAUNCH_GEMM(BM_, BN_, WM_, WN_, GX, GY)                                                                        \
  do {                                                                                                                   \
    dim3 grid(GX, GY, zdim);                                                                                             \
    if constexpr (WM_ * WN_ != 4) {                                                                                      \
      LAUNCH_GEMM_RS(BM_, BN_, WM_, WN_);                                                                                \
    } else if (K >= 1024) {                                                                                              \
      LAUNCH_GEMM_RS(BM_, BN_, WM_, WN_);                                                                                \
    } else if (K >= 128) hipLaunchKernelGGL((k_gemm<BM_, BN_, WM_, WN_, 64, AL, EP>), grid, blk, 0, c->stream, al, Bm, ldb, N, ep); \
    else hipLaunchKernelGGL((k_gemm<BM_, BN_, WM_, WN_, 32, AL, EP>), grid, blk, 0, c->stream, al, Bm, ldb, N, ep);        \
  } while (0)
  if (N > 64) {
    if (K >= 1024 && (int64_t)cdiv(M, 256) * cdiv(N, 128) * zdim >= 256) LAUNCH_GEMM(256, 128, 4, 2, cdiv(M, 256), cdiv(N, 128));
    else if ((int64_t)cdiv(M, 128) * cdiv(N, 128) * zdim >= 256 || M <= 64) LAUNCH_GEMM(128, 128, 2, 2, cdiv(M, 128), cdiv(N, 128));
    else LAUNCH_GEMM(64, 64, 2, 2, cdiv(M, 64), cdiv(N, 64));
  } else if (N > 32) {
    if ((int64_t)cdiv(M, 128) * zdim >= 256 || M <= 64) LAUNCH_GEMM(128, 64, 2, 2, cdiv(M, 128), 1);
    else LAUNCH_GEMM(64, 64, 2, 2, cdiv(M, 64), 1);
  } else {
    LAUNCH_GEMM(128, 32, 4, 1, cdiv(M, 128), 1);
  }
#undef LAUNCH_GEMM
#undef LAUNCH_GEMM_RS
  LAUNCHCHK(c, what);
  return PPO_OK;
}

ImgAddr plain_rows(const bf16_t* base, int64_t ld) { ImgAddr a; a.base = base; a.idx = nullptr; a.stride_b = ld; a.stride_v = 0; a.V = 1; return a; }
ARows plain_arows(const bf16_t* base, int64_t ld, int M, int K) {
  ARows r; r.a = plain_rows(base, ld); r.HW = 1; r.C = 0; r.M = M; r.K = K; r.plain = true; return r;
}
MapRows plain_map(int64_t ld, int M) { MapRows m; m.stride_b = ld; m.stride_v = 0; m.V = 1; m.HW = 1; m.C = 0; m.M = M; return m; }

// All queued partial-sum reductions in one launch; the partial workspaces are free again afterwards.
int flush_reduces(Ctx* c) {
  ReduceJobs& J = c->rjobs;
  if (J.njobs > 0 || c->lossfin.on) {
    double bytes = 0.0;
    for (int j = 0; j < J.njobs; ++j) bytes += 4.0 * ((double)J.splits[j] + 1.0) * (double)J.n[j];
    ProfScope ps(c, "wgrad_reduce", 0.0, bytes);
    for (int j = J.njobs; j <= ReduceJobs::MAXJ; ++j) J.first[j] = c->rjob_blocks;
    hipLaunchKernelGGL(k_reduce_batch, dim3(c->rjob_blocks + (c->lossfin.on ? 1 : 0)), dim3(256), 0, c->stream, J, c->lossfin);
    LAUNCHCHK(c, "k_reduce_batch");
    c->lossfin.on = 0;
  }
  J.njobs = 0; c->rjob_blocks = 0;
  c->partial = c->partial_base; c->partial_elems = c->partial_cap;
  c->bias_partial = c->bias_partial_base; c->bias_partial_elems = c->bias_partial_cap;
  return PPO_OK;
}
// Make room for a kernel that would like `need` partial and `bneed` bias-partial elements.
int ensure_partial(Ctx* c, int64_t need, int64_t bneed) {
  if (need > c->partial_elems || bneed > c->bias_partial_elems || c->rjobs.njobs + 2 > ReduceJobs::MAXJ) return flush_reduces(c);
  return PPO_OK;
}
// Queue the reduction of `splits` partials of n elements that start at the cursor (kind as in ReduceJobs) and
// move the cursor behind them; with bias: the same for `splits` bias partials of nb elements (plain sums).
void defer_reduce(Ctx* c, int kind, int splits, int64_t n, int N, int K, float* dst, float* dst2, bool accumulate, bool with_bias, int64_t nb, float* bdst) {
  ReduceJobs& J = c->rjobs;
  auto add = [&](int kd, const float* part, int64_t nn, float* d, float* d2) {
    const int j = J.njobs++;
    J.first[j] = c->rjob_blocks; J.kind[j] = kd; J.splits[j] = splits; J.N[j] = N; J.K[j] = K; J.accumulate[j] = accumulate ? 1 : 0;
    J.n[j] = nn; J.partial[j] = part; J.dst[j] = d; J.dst2[j] = d2;
    J.vec[j] = (nn % 4 == 0 && (reinterpret_cast<uintptr_t>(part) & 15) == 0) ? 1 : 0;
    c->rjob_blocks += cdiv(nn, J.vec[j] ? 128 : 32);
  };
  add(kind, c->partial, n, dst, dst2);
  c->partial += (int64_t)splits * n; c->partial_elems -= (int64_t)splits * n;
  if (with_bias) {
    add(0, c->bias_partial, nb, bdst, nullptr);
    c->bias_partial += (int64_t)splits * nb; c->bias_partial_elems -= (int64_t)splits * nb;
  }
}

// Wide plain weight gradient through the LDS-ring kernel (wgrad_rs.hip.h); returns 1 when the shape is not covered.
int launch_wgrad_rs(Ctx* c, const bf16_t* dy, int64_t ld_dy, const bf16_t* x, int64_t ld_x, int Nn, int Kk, int M, float* gw, float* gb, bool accumulate,
                    const std::string& name, double abytes) {
  typedef WgradRsShape S;
  if (Nn < 128 || Kk < 1024 || Nn % 8 || Kk % 8 || ld_dy % 8 || ld_x % 8 || M < 128) return 1;
  const int tiles = cdiv(Kk, S::TK) * cdiv(Nn, S::TN);
  // few splits (their fp32 partials cost traffic), but enough blocks to fill the chip's 256 CUs in whole rounds
  int splits = 1;
  double best = 0.0;
  for (int sp = 1; sp <= 8; ++sp) {
    if (cdiv(M, sp) < 512 && sp > 1) break;
    const int blocks = tiles * sp;
    const double eff = (double)blocks / (double)(cdiv(blocks, 256) * 256) - 0.06 * (sp - 1);
    if (eff > best + 1e-9) { best = eff; splits = sp; }
  }
  const int64_t per = (int64_t)Nn * Kk;
  if (splits > 1) { const int erc = ensure_partial(c, (int64_t)splits * per, gb ? (int64_t)splits * Nn : 0); if (erc) return erc; }
  if (splits > 1 && ((int64_t)splits * per > c->partial_elems || (gb && (int64_t)splits * Nn > c->bias_partial_elems))) splits = 1;
  int rows = cdiv(M, splits);
  rows = (rows + S::ROWS - 1) / S::ROWS * S::ROWS;
  splits = cdiv(M, rows);
  WgradRsArgs a;
  a.dy = dy; a.ld_dy = ld_dy; a.x = x; a.ld_x = ld_x; a.M = M; a.Nn = Nn; a.Kk = Kk; a.rows_per_split = rows; a.zpage = c->zpage;
  a.direct = splits == 1 ? 1 : 0; a.accumulate = accumulate ? 1 : 0;
  a.out = a.direct ? gw : c->partial; a.bias_out = gb ? (a.direct ? gb : c->bias_partial) : nullptr;
  {
    ProfScope ps(c, name, 2.0 * M * (double)Nn * Kk, abytes);
    static uint64_t attr_devs = 0;  /* bit d: set on device d */
    if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)k_wgrad_rs, hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS_BYTES)); attr_devs |= 1ull << c->dev; }
    hipLaunchKernelGGL(k_wgrad_rs, dim3(cdiv(Kk, S::TK), cdiv(Nn, S::TN), splits), dim3(S::THREADS), S::LDS_BYTES, c->stream, a);
    LAUNCHCHK(c, "k_wgrad_rs");
  }
  if (splits > 1) defer_reduce(c, 0, splits, per, 0, 0, gw, nullptr, accumulate, gb != nullptr, Nn, gb);
  return PPO_OK;
}

// G[Nn][Kk] (+)= Dy^T * A over M rows, plus optional bias gradient gb[Nn].
template <class DL, class AL>
int launch_wgrad(Ctx* c, const DL& dl_, const AL& al_, int Nn, int Kk, int M, float* gw, float* gb, bool accumulate, const std::string& name, double abytes) {
  if (M <= 0) return PPO_OK;
  if constexpr (std::is_same<DL, ARows>::value && std::is_same<AL, ARows>::value) {
    if (dl_.plain && al_.plain) {
      const int rc = launch_wgrad_rs(c, dl_.a.base, dl_.a.stride_b, al_.a.base, al_.a.stride_b, Nn, Kk, M, gw, gb, accumulate, name, abytes);
      if (rc != 1) return rc;
    }
  }
  DL dl = dl_; AL al = al_;
  dl.prepare(); al.prepare();
  const char* what = name.c_str();
  // wide outputs (the first hidden layer) have enough tiles with narrow blocks and few splits: the fp32 partials,
  // not the operands, are then the larger part of the traffic
  const int ktw = Kk <= 128 ? 1 : (Kk <= 256 ? 2 : (Kk >= 1024 ? 1 : 3));
  const int tiles = cdiv(Kk, 128 * ktw) * cdiv(Nn, 64);
  int splits = cdiv(Kk >= 1024 ? 512 : 768, tiles);
  const int max_by_rows = cdiv(M, 128);
  if (splits > max_by_rows) splits = max_by_rows;
  const int64_t per = (int64_t)Nn * Kk;
  { const int erc = ensure_partial(c, (int64_t)splits * per, (int64_t)splits * Nn); if (erc) return erc; }
  if ((int64_t)splits * per > c->partial_elems) splits = (int)(c->partial_elems / per);
  if ((int64_t)splits * Nn > c->bias_partial_elems) splits = (int)(c->bias_partial_elems / Nn);
  if (splits < 1) return fail(c, PPO_ENOMEM, "weight-gradient workspace too small for %s", what);
  int rows = cdiv(M, splits);
  rows = (rows + 31) / 32 * 32;
  splits = cdiv(M, rows);
  dim3 grid(cdiv(Kk, 128 * ktw), cdiv(Nn, 64), splits);
  {
    ProfScope ps(c, name, 2.0 * M * (double)Nn * Kk, abytes);
    float* bp = gb ? c->bias_partial : nullptr;
    if (ktw == 1) hipLaunchKernelGGL((k_wgrad<1, DL, AL>), grid, dim3(256), 0, c->stream, dl, al, Nn, Kk, M, rows, c->partial, bp);
    else if (ktw == 2) hipLaunchKernelGGL((k_wgrad<2, DL, AL>), grid, dim3(256), 0, c->stream, dl, al, Nn, Kk, M, rows, c->partial, bp);
    else hipLaunchKernelGGL((k_wgrad<3, DL, AL>), grid, dim3(256), 0, c->stream, dl, al, Nn, Kk, M, rows, c->partial, bp);
    LAUNCHCHK(c, what);
  }
  defer_reduce(c, 0, splits, per, 0, 0, gw, nullptr, accumulate, gb != nullptr, Nn, gb);
  return PPO_OK;
}

// bf16 copies of the parameters in the layouts the backward GEMMs read
// Parity-class-packed transposed-conv weights of layer l for the implicit-GEMM paths: rebuilt when they
// are first needed after a change of the weights (the LDS-image kernels use the per-tap transposes instead).
int ensure_packed_dgrad_weights(Ctx* c, int l) {
  if (c->wd_ver[l] == c->wver) return PPO_OK;
  const int Co = c->cC[l + 1], Ci = c->cC[l];
  for (int py = 0; py < 2; ++py) {
    int64_t n = (int64_t)2 * Ci * (1 + py) * 2 * Co;
    hipLaunchKernelGGL(k_pack_dgrad_w, dim3(cdiv(n, 256)), dim3(256), 0, c->stream, c->shadow + c->convW[l], Co, Ci, py, c->wd[l][py]);
  }
  LAUNCHCHK(c, "k_pack_dgrad_w");
  c->wd_ver[l] = c->wver;
  return PPO_OK;
}

int repack_weights(Ctx* c) {
  c->wver += 1;
  ProfScope ps(c, "weight_repack", 0.0, 4.0 * (double)c->total);
  RepackJobs jobs;
  int nj = 0, nblocks = 0;
  auto add = [&](int kind, const bf16_t* src, bf16_t* dst, int a, int b, int ld, int64_t elems) {
    jobs.first[nj] = nblocks; jobs.kind[nj] = kind; jobs.src[nj] = src; jobs.dst[nj] = dst; jobs.a[nj] = a; jobs.b[nj] = b; jobs.ld[nj] = ld;
    nblocks += cdiv(elems, 256); ++nj;
  };
  if (c->nconv - 1 + c->nfc + 1 + (c->XH > 0 ? 2 : 0) + (c->E > 0 ? 1 : 0) + c->nl > RepackJobs::MAXJ) return fail(c, PPO_ESHAPE, "too many layers for one re-pack launch");
  for (int l = 1; l < c->nconv; ++l)
    add(1, c->shadow + c->convW[l], c->wtap[l], c->cC[l + 1], c->cC[l], 0, (int64_t)9 * c->cC[l] * c->cC[l + 1]);
  for (int l = 0; l < c->nfc; ++l)
    add(0, c->shadow + c->fcW[l], c->fcT[l], c->fout[l], c->fin[l], c->fout[l], (int64_t)c->fin[l] * c->fout[l]);
  add(0, c->shadow + c->headW, c->headT, c->NH, c->hid, HEAD_LD, (int64_t)c->hid * HEAD_LD);
  if (c->XH > 0) {
    add(0, c->shadow + c->aux1W, c->aux1T, c->XH, c->hid, c->XH, (int64_t)c->hid * c->XH);
    add(0, c->shadow + c->aux2W, c->aux2T, c->X, c->XH, HEAD_LD, (int64_t)c->XH * HEAD_LD);
  }
  if (c->E > 0) add(0, c->shadow + c->embW, c->embT, c->E, c->flat, c->E, (int64_t)c->flat * c->E);
  for (int l = 0; l < c->nl; ++l)
    add(0, c->shadow + c->lstmW[l], c->lstmWT[l], 4 * c->H, c->lin[l] + c->H, 4 * c->H, (int64_t)(c->lin[l] + c->H) * 4 * c->H);
  jobs.first[nj] = nblocks; jobs.njobs = nj;
  for (int j = nj + 1; j <= RepackJobs::MAXJ; ++j) jobs.first[j] = nblocks;
  for (int j = nj; j < RepackJobs::MAXJ; ++j) { jobs.kind[j] = 0; jobs.src[j] = nullptr; jobs.dst[j] = nullptr; jobs.a[j] = jobs.b[j] = jobs.ld[j] = 0; }
  hipLaunchKernelGGL(k_repack_all, dim3(nblocks + (c->gnfin.on ? 1 : 0)), dim3(256), 0, c->stream, jobs, c->gnfin);
  LAUNCHCHK(c, "weight repack");
  c->gnfin.on = 0;
  return PPO_OK;
}

int refresh_shadow(Ctx* c) {
  hipLaunchKernelGGL(k_cast_bf16, dim3(cdiv(c->total, 256)), dim3(256), 0, c->stream, c->p, c->shadow, c->total);
  LAUNCHCHK(c, "k_cast_bf16");
  return repack_weights(c);
}

ImgAddr conv_out_addr(Ctx* c, int l, const bf16_t* contiguous, const bf16_t* strided) {
  // output of conv layer l (0-based) for a chunk: the last layer lives inside the feature matrix
  ImgAddr a; a.idx = nullptr; a.V = c->V;
  if (l == c->nconv - 1) { a.base = strided; a.stride_b = c->feat_ld; a.stride_v = c->flat; }
  else { int64_t e = (int64_t)c->cC[l + 1] * c->cH[l + 1] * c->cW[l + 1]; a.base = contiguous; a.stride_b = e * c->V; a.stride_v = e; }
  return a;
}

// Forward convolution through the LDS-image kernel; returns 1 when the layer's shape is not one
// it covers (the caller then takes the implicit-GEMM path).
template <int CIN, int WIDE>
int launch_conv_fwd_tile_t(Ctx* c, ConvTileArgs a, const std::string& name, double flops, double abytes) {
  typedef ConvTileShape<CIN, WIDE> S;
  const int segs = cdiv(a.W * S::PIX, 1024), ni = cdiv(2 * a.TR + 1, 4) * segs;  // loads per loader wave per band
  // as many ring images as fit: a loader wave has (nbuf - 2) * ni loads outstanding behind the band it waits for
  a.nbuf = S::MAXBUF;
  while (a.nbuf > 3 && (S::lds_bytes(a.W, a.TR, a.nbuf) > 160 * 1024 || (a.nbuf - 2) * ni > 63)) --a.nbuf;
  const int lds = S::lds_bytes(a.W, a.TR, a.nbuf);
  if (segs > S::MAXSEG || ni > 63 || lds > 160 * 1024) return 1;
  const int gy = cdiv(a.Cout, S::BN);
  int gx = 256 / gy; if (gx > a.ntiles) gx = a.ntiles; if (gx < 1) gx = 1;
  // bands of four or more output rows share at most an eighth of their input rows with a neighbour: read once, non-temporal
  const bool nt = a.TR >= 4;
  auto kfn = nt ? k_conv_fwd_tile<CIN, LOAD_NT, WIDE> : k_conv_fwd_tile<CIN, 0, WIDE>;
  static uint64_t attr_devs[2] = {0, 0};  // bit d: set on device d
  if (!((attr_devs[nt] >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_devs[nt] |= 1ull << c->dev; }
  ProfScope ps(c, name, flops, abytes);
  hipLaunchKernelGGL(kfn, dim3(gx, gy), dim3(S::THREADS), lds, c->stream, a);
  LAUNCHCHK(c, "k_conv_fwd_tile");
  return PPO_OK;
}
int launch_conv_fwd_tile(Ctx* c, const AConvFwd& al, const ImgAddr& o, int Cout, const bf16_t* w, const float* bias, int nimg,
                         const std::string& name, double abytes, uint32_t* bits) {
  if ((al.Cin != 32 && al.Cin != 64) || Cout % 8 || nimg < 1 || al.in.idx) return 1;
  const int BM = al.Cin == 32 ? 128 : 64;
  if (al.Wo > BM) return 1;
  ConvTileArgs a;
  a.in = al.in; a.in.prepare();
  a.out = const_cast<bf16_t*>(o.base); a.out_stride_b = o.stride_b; a.out_stride_v = o.stride_v;
  a.w = w; a.bias = bias; a.zpage = c->zpage; a.bits = bits; a.V = o.V; a.H = al.H; a.W = al.W; a.Ho = al.Ho; a.Wo = al.Wo; a.Cout = Cout;
  const int trmax = BM / al.Wo < al.Ho ? BM / al.Wo : al.Ho;
  a.NB = cdiv(al.Ho, trmax); a.TR = cdiv(al.Ho, a.NB);  // balanced bands
  a.ntiles = nimg * a.NB; a.nbuf = 3;
  const double flops = 2.0 * (double)al.M * Cout * al.K;
  if (al.Cin == 32) return launch_conv_fwd_tile_t<32, 0>(c, a, name, flops, abytes);
  // more than 64 output channels: the 64 x 128 form reads the input once
  return Cout > 64 ? launch_conv_fwd_tile_t<64, 1>(c, a, name, flops, abytes) : launch_conv_fwd_tile_t<64, 0>(c, a, name, flops, abytes);
}

// Weight (and bias) gradient of conv layer with 32 or 64 input channels through the LDS-image
// kernel; returns 1 when the shape is not covered (the caller then takes the implicit-GEMM path).
template <int CIN>
int launch_conv_wgrad_tile_t(Ctx* c, ConvWgradArgs a, float* gw, float* gb, bool accumulate, const std::string& name, double flops, double abytes) {
  typedef ConvWgradShape<CIN> S;
  // largest band that fits the pixel-step table and three ring buffers, then balanced over the image
  int TR = 0;
  for (int tr = a.Ho; tr >= 1; --tr)
    if (tr * a.Wo <= 16 * S::MAXSTEP && S::lds_bytes(a.W, tr, cdiv(tr * a.Wo, 16), 3) <= 158 * 1024) { TR = tr; break; }
  if (TR == 0) return 1;
  a.NB = cdiv(a.Ho, TR); a.TR = cdiv(a.Ho, a.NB); a.nstep = cdiv(a.TR * a.Wo, 16);
  const int nimg = a.ntiles;  // passed in as the image count
  a.ntiles = nimg * a.NB;
  const int segs = cdiv(a.W * S::PIX, 1024), ni = cdiv(2 * a.TR + 1, 4) * segs + cdiv(a.nstep * 2, 4);  // loads per loader wave per band
  if (segs > S::MAXSEG || ni > 63) return 1;
  a.nbuf = S::MAXBUF;  // as many ring buffers as fit (the balanced band may be smaller than the largest that fits three)
  while (a.nbuf > 3 && (S::lds_bytes(a.W, a.TR, a.nstep, a.nbuf) > 158 * 1024 || (a.nbuf - 2) * ni > 63)) --a.nbuf;
  const int gy = cdiv(a.Cout, 64), K = 9 * CIN;
  int gx = 256 / gy; if (gx > a.ntiles) gx = a.ntiles; if (gx < 1) gx = 1;
  const int64_t per = (int64_t)a.Cout * K;
  { const int erc = ensure_partial(c, (int64_t)gx * per, gb ? (int64_t)gx * a.Cout : 0); if (erc) return erc; }
  if ((int64_t)gx * per > c->partial_elems) gx = (int)(c->partial_elems / per);
  if (gb && (int64_t)gx * a.Cout > c->bias_partial_elems) gx = (int)(c->bias_partial_elems / a.Cout);
  if (gx < 1) return 1;
  a.partial = c->partial; a.bias_partial = gb ? c->bias_partial : nullptr;
  const int lds = S::lds_bytes(a.W, a.TR, a.nstep, a.nbuf);
  // the step counts of the benchmark shapes have a form of their own (branch-free tile loop); index 0: any count
  constexpr int NS1 = S::MAXSTEP, NS2 = S::MAXSTEP - 1;
  const int form = a.nstep == NS1 ? 1 : (a.nstep == NS2 ? 2 : 0);
  auto kfn = form == 1 ? k_conv_wgrad_tile<CIN, NS1> : (form == 2 ? k_conv_wgrad_tile<CIN, NS2> : k_conv_wgrad_tile<CIN, 0>);
  static uint64_t attr_devs[3] = {0, 0, 0};  /* bit d: set on device d */
  if (!((attr_devs[form] >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_devs[form] |= 1ull << c->dev; }
  {
    ProfScope ps(c, name, flops, abytes);
    hipLaunchKernelGGL(kfn, dim3(gx, gy), dim3(S::THREADS), lds, c->stream, a);
    LAUNCHCHK(c, "k_conv_wgrad_tile");
  }
  defer_reduce(c, 1, gx, per, a.Cout, K, gw, nullptr, accumulate, gb != nullptr, a.Cout, gb);
  return PPO_OK;
}
int launch_conv_wgrad_tile(Ctx* c, const ImgAddr& dy, const AConvFwd& xl, int Cout, int nimg, float* gw, float* gb, bool accumulate,
                           const std::string& name, double abytes) {
  if ((xl.Cin != 32 && xl.Cin != 64) || Cout % 8 || nimg < 1 || xl.in.idx || dy.idx) return 1;
  ConvWgradArgs a;
  a.in = xl.in; a.in.prepare(); a.dy = dy; a.dy.prepare(); a.zpage = c->zpage; a.partial = nullptr; a.bias_partial = nullptr;
  a.H = xl.H; a.W = xl.W; a.Ho = xl.Ho; a.Wo = xl.Wo; a.Cout = Cout; a.TR = 0; a.NB = 0; a.nstep = 0; a.nbuf = 3;
  a.ntiles = nimg;  // image count; the template turns it into tiles
  const double flops = 2.0 * (double)xl.M * Cout * xl.K;
  return xl.Cin == 32 ? launch_conv_wgrad_tile_t<32>(c, a, gw, gb, accumulate, name, flops, abytes)
                      : launch_conv_wgrad_tile_t<64>(c, a, gw, gb, accumulate, name, flops, abytes);
}

// Transposed convolution through the quad-organised LDS-image kernel; returns 1 when the shape is
// not covered (the caller then takes the implicit-GEMM path).  With C0 > 0 the kernel also forms
// the first layer's weight-gradient partials (a.img0, a.H0, a.W0 set by the caller) and *grid_out
// receives the number of partials.
template <int CI, int C0>
int launch_conv_dgrad_tile_t(Ctx* c, ConvDgradArgs a, int nimg, const std::string& name, double flops, double abytes, int* grid_out) {
  typedef ConvDgradShape<CI> S;
  if (a.Wo > S::BQ) return 1;
  auto lds_of = [&](int tq) { return S::lds_bytes(a.W, a.Wo, tq) + (C0 > 0 ? S::fused_extra(a.W, a.W0, C0, tq) : 0); };
  auto fits = [&](int tq) {
    if (S::stage_bytes(a.W, tq) > S::MAXCH * 256 * 16 || lds_of(tq) > 158 * 1024) return false;
    if (C0 > 0 && ((tq * a.W) % 2 != 0 || tq * a.W / 2 > 128)) return false;  // pixels per finishing wave: two per lane at most
    return true;
  };
  int TQ = S::BQ / a.Wo < a.Ho ? S::BQ / a.Wo : a.Ho;
  while (TQ > 1 && !fits(TQ)) --TQ;
  if (!fits(TQ)) return 1;
  a.NB = cdiv(a.Ho, TQ);
  if (C0 == 0 || fits(cdiv(a.Ho, a.NB))) TQ = cdiv(a.Ho, a.NB);  // balanced bands
  a.TQ = TQ; a.NB = cdiv(a.Ho, TQ); a.ntiles = nimg * a.NB;
  const int segs = cdiv(a.Wo * 128, 1024);
  int ni = cdiv(a.TQ + 1, 2) * segs;
  if (C0 > 0) {
    const int rb0 = a.W0 * C0 * 2;
    if (rb0 % 16) return 1;
    ni += cdiv(cdiv((4 * a.TQ + 1) * rb0, 1024), 2);
  }
  if (segs > S::MAXSEG || ni > 63) return 1;
  int gx = a.ntiles < 256 ? a.ntiles : 256;
  if (C0 > 0) {
    const int64_t npair = (int64_t)CI * (9 * C0 + 1);
    { const int erc = ensure_partial(c, gx * npair, 0); if (erc) return erc; }
    if (gx * npair > c->partial_elems) gx = (int)(c->partial_elems / npair);
    if (gx < 1) return 1;
    a.partial0 = c->partial;
    *grid_out = gx;
  }
  auto kfn = k_conv_dgrad_tile<CI, C0>;
  static uint64_t attr_devs = 0;  /* bit d: set on device d */
  if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_devs |= 1ull << c->dev; }
  ProfScope ps(c, name, flops, abytes);
  hipLaunchKernelGGL(kfn, dim3(gx), dim3(S::THREADS), lds_of(a.TQ), c->stream, a);
  LAUNCHCHK(c, "k_conv_dgrad_tile");
  return PPO_OK;
}
ConvDgradArgs conv_dgrad_args(Ctx* c, const ImgAddr& dy, const ImgAddr& xa, const uint32_t* xbits, bf16_t* dx, const bf16_t* wt, int H, int W, int Ho, int Wo) {
  ConvDgradArgs a;
  a.dy = dy; a.dy.prepare(); a.dx = dx; a.xbits = xbits; a.x_stride_b = xa.stride_b; a.x_stride_v = xa.stride_v;
  a.wt = wt; a.zpage = c->zpage; a.V = xa.V; a.H = H; a.W = W; a.Ho = Ho; a.Wo = Wo; a.TQ = 0; a.NB = 0; a.ntiles = 0; a.seg_split = 0;
  a.img0 = ImgAddr(); a.img0.base = nullptr; a.img0.idx = nullptr; a.img0.stride_b = 0; a.img0.stride_v = 0; a.img0.V = 1;
  a.H0 = 0; a.W0 = 0; a.partial0 = nullptr;
  return a;
}
// The form for 128 gradient channels and 64 result channels (the contraction split over two pairs of compute waves).
int launch_conv_dgrad_k2_tile(Ctx* c, ConvDgradArgs a, int nimg, const std::string& name, double flops, double abytes) {
  typedef ConvDgradK2Shape S;
  if (a.Wo > S::BQ) return 1;
  auto fits = [&](int tq) { return S::stage_bytes(a.W, tq) <= S::MAXCH * S::NFT * 16 && S::lds_bytes(a.W, a.Wo, tq) <= 158 * 1024; };
  int TQ = S::BQ / a.Wo < a.Ho ? S::BQ / a.Wo : a.Ho;
  while (TQ > 1 && !fits(TQ)) --TQ;
  if (!fits(TQ)) return 1;
  a.NB = cdiv(a.Ho, TQ); TQ = cdiv(a.Ho, a.NB);  // balanced bands (fewer, larger tiles beat fuller ones: the cost of a tile is mostly fixed)
  a.TQ = TQ; a.NB = cdiv(a.Ho, TQ); a.ntiles = nimg * a.NB;
  const int segs = cdiv(a.Wo * S::PB, 1024);
  if (segs > S::MAXSEG || (a.TQ + 1) * segs > 63) return 1;
  const int gx = a.ntiles < 256 ? a.ntiles : 256;
  auto kfn = k_conv_dgrad_k2_tile;
  static uint64_t attr_devs = 0;  /* bit d: set on device d */
  if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_devs |= 1ull << c->dev; }
  ProfScope ps(c, name, flops, abytes);
  hipLaunchKernelGGL(kfn, dim3(gx), dim3(S::THREADS), S::lds_bytes(a.W, a.Wo, a.TQ), c->stream, a);
  LAUNCHCHK(c, "k_conv_dgrad_k2_tile");
  return PPO_OK;
}
int launch_conv_dgrad_tile(Ctx* c, const ImgAddr& dy, const ImgAddr& xa, const uint32_t* xbits, bf16_t* dx, const bf16_t* wt, int Co, int Ci, int H, int W, int Ho, int Wo,
                           int nimg, const std::string& name, double flops, double abytes) {
  if (Co == 128 && Ci == 64 && !dy.idx && nimg >= 1 && xbits) {
    ConvDgradArgs a2 = conv_dgrad_args(c, dy, xa, xbits, dx, wt, H, W, Ho, Wo);
    return launch_conv_dgrad_k2_tile(c, a2, nimg, name, flops, abytes);
  }
  if (Co != 64 || (Ci != 32 && Ci != 64) || dy.idx || nimg < 1 || !xbits) return 1;
  ConvDgradArgs a = conv_dgrad_args(c, dy, xa, xbits, dx, wt, H, W, Ho, Wo);
  return Ci == 32 ? launch_conv_dgrad_tile_t<32, 0>(c, a, nimg, name, flops, abytes, nullptr)
                  : launch_conv_dgrad_tile_t<64, 0>(c, a, nimg, name, flops, abytes, nullptr);
}
// Register-fused form of the same pair of layers (conv_dgrad_wgrad0_tile.hip.h); returns 1 when the shape is not covered.
template <int C0, int NCW, int WC = 0>
int launch_conv_dgrad_wgrad0_reg_t(Ctx* c, ConvDgradArgs a, int nimg, const std::string& name, double flops, double abytes, int* grid_out) {
  typedef ConvDgradW0Shape<NCW> S;
  if (WC && a.W != WC) return 1;
  constexpr bool ones = C0 == 1 && WC != 0;  // the kernel's ONES
  const int rb0 = a.W0 * C0 * 2;
  if (a.W % 8 || rb0 % 16 || a.Wo * 2 != a.W || a.Wo > S::BQ || a.H != (a.H0 + 1) / 2 || a.W * 2 != a.W0) return 1;
  auto fits = [&](int tq) {
    return tq * a.Wo <= S::BQ && S::lds_bytes(a.W, a.Wo, a.W0, C0, tq, ones) <= 160 * 1024 && S::loads_fit(a.W, a.Wo, a.W0, C0, tq) &&
           S::dyimg_bytes(a.Wo, tq) <= 65536;  // offsets into the page of zeros
  };
  int TQ = S::BQ / a.Wo < a.Ho ? S::BQ / a.Wo : a.Ho;
  while (TQ > 1 && !fits(TQ)) --TQ;
  if (TQ < 1 || !fits(TQ)) return 1;
  a.NB = cdiv(a.Ho, TQ); a.TQ = cdiv(a.Ho, a.NB); a.NB = cdiv(a.Ho, a.TQ); a.ntiles = nimg * a.NB;
  a.dv_rb0 = make_fastdiv(rb0); a.dv_mrow = make_fastdiv(a.W * 4); a.seg_split = S::seg_split(a.Wo, a.TQ);
  int gx = a.ntiles < 256 ? a.ntiles : 256;
  const int64_t npair = (int64_t)S::CI * (9 * C0 + 1);
  { const int erc = ensure_partial(c, gx * npair, 0); if (erc) return erc; }
  if (gx * npair > c->partial_elems) gx = (int)(c->partial_elems / npair);
  if (gx < 1) return 1;
  a.partial0 = c->partial;
  *grid_out = gx;
  auto kfn = k_conv_dgrad_wgrad0_tile<C0, NCW, WC>;
  static uint64_t attr_devs = 0;  /* bit d: set on device d */
  if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024)); attr_devs |= 1ull << c->dev; }
  ProfScope ps(c, name, flops, abytes);
  hipLaunchKernelGGL(kfn, dim3(gx), dim3(S::THREADS), S::lds_bytes(a.W, a.Wo, a.W0, C0, a.TQ, ones), c->stream, a);
  LAUNCHCHK(c, "k_conv_dgrad_wgrad0_tile");
  return PPO_OK;
}
// The same with the first layer's weight gradient fused in (depth or RGB input, 32 channels after the first layer).
int launch_conv_dgrad_wgrad0_tile(Ctx* c, const ImgAddr& dy, const ImgAddr& xa, const uint32_t* xbits, const bf16_t* wt, int Co, int Ci, int H, int W, int Ho, int Wo,
                                  const ImgAddr& img0, int C0, int H0, int W0, int nimg, const std::string& name, double flops, double abytes, int* grid_out) {
  if (Co != 64 || Ci != 32 || (C0 != 1 && C0 != 3) || dy.idx || nimg < 1 || !xbits) return 1;
  ConvDgradArgs a = conv_dgrad_args(c, dy, xa, xbits, nullptr, wt, H, W, Ho, Wo);
  a.img0 = img0; a.img0.prepare(); a.H0 = H0; a.W0 = W0;
  // eight compute waves (two per SIMD) when the larger tile fits, else four
  // (the 80-wide result of 120x160 depth images has a form of its own with the row pitches known at compile time)
  int rrc = C0 == 1 ? launch_conv_dgrad_wgrad0_reg_t<1, 8, 80>(c, a, nimg, name, flops, abytes, grid_out) : 1;
  if (rrc == 1)
    rrc = C0 == 1 ? launch_conv_dgrad_wgrad0_reg_t<1, 8>(c, a, nimg, name, flops, abytes, grid_out)
                  : launch_conv_dgrad_wgrad0_reg_t<3, 8>(c, a, nimg, name, flops, abytes, grid_out);
  if (rrc == 1)
    rrc = C0 == 1 ? launch_conv_dgrad_wgrad0_reg_t<1, 4>(c, a, nimg, name, flops, abytes, grid_out)
                  : launch_conv_dgrad_wgrad0_reg_t<3, 4>(c, a, nimg, name, flops, abytes, grid_out);
  if (rrc != 1) return rrc;
  return C0 == 1 ? launch_conv_dgrad_tile_t<32, 1>(c, a, nimg, name, flops, abytes, grid_out)
                 : launch_conv_dgrad_tile_t<32, 3>(c, a, nimg, name, flops, abytes, grid_out);
}

// First convolution forward through the LDS-ring kernel; returns 1 when the shape is not covered.
template <int C0>
int launch_conv0_fwd_tile_t(Ctx* c, Conv0Args a, int nimg) {
  typedef Conv0Shape<C0> S;
  const int rb = a.W * C0 * 2;
  if (rb % 16 || ((int64_t)a.H * rb) % 16 || a.Cout % 8 || a.Cout > 64) return 1;
  int TR = 0;
  for (int tr = a.Ho; tr >= 1; --tr)
    if (cdiv((2 * tr + 1) * rb, 1024) <= 63 && tr * a.Wo <= 1024 && S::lds_bytes(a.W, tr, a.Cout) <= 64 * 1024) { TR = tr; break; }
  if (TR == 0) return 1;
  a.NB = cdiv(a.Ho, TR); a.TR = cdiv(a.Ho, a.NB); a.ntiles = nimg * a.NB;
  a.dv_wo = make_fastdiv(a.Wo);
  int gx = a.ntiles < 512 ? a.ntiles : 512;
  a.tile_blocks = gx;
  if (a.gather_blocks > 0) a.gather_blocks = (int)std::min<int64_t>(32, cdiv((int64_t)a.pB * a.P, 512));
  auto kfn = k_conv0_fwd_tile<C0>;
  static uint64_t attr_devs = 0;  /* bit d: set on device d */
  if (!((attr_devs >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024)); attr_devs |= 1ull << c->dev; }
  hipLaunchKernelGGL(kfn, dim3(gx + a.gather_blocks), dim3(S::THREADS), S::lds_bytes(a.W, a.TR, a.Cout), c->stream, a);
  LAUNCHCHK(c, "k_conv0_fwd_tile");
  return PPO_OK;
}

// The student's auxiliary MLP head on the last hidden layer x [n][hid]: hidden layer (bias, ReLU) into auxact, its
// X outputs into the columns [A_main, A) of the head-output rows, behind the linear head's.
int aux_head_forward(Ctx* c, const bf16_t* x, int64_t ldx, int n) {
  if (c->XH <= 0) return PPO_OK;
  ARows al = plain_arows(x, ldx, n, c->hid);
  Ep<MapRows, bf16_t, true, true, false> e1;
  e1.map = plain_map(c->XH, n); e1.out = c->auxact; e1.bias = c->p + c->aux1B; e1.mask = nullptr; e1.N = c->XH;
  int rc = launch_gemm(c, al, n, c->shadow + c->aux1W, c->hid, c->XH, c->hid, e1, "aux_fwd.0", 2.0 * n * ((double)c->hid + c->XH) + 2.0 * c->hid * c->XH);
  if (rc) return rc;
  ARows a2 = plain_arows(c->auxact, c->XH, n, c->XH);
  Ep<MapRows, float, true, false, false> e2;
  e2.map = plain_map(HEAD_LD, n); e2.out = c->headout + c->A_main; e2.bias = c->p + c->aux2B; e2.mask = nullptr; e2.N = c->X;
  return launch_gemm(c, a2, n, c->shadow + c->aux2W, c->XH, c->X, c->XH, e2, "aux_fwd.1", 2.0 * n * c->XH + 4.0 * n * c->X);
}
// Its backward from the loss gradient rows dhead [n][32]: weight and bias gradients of both layers, and the
// gradient it sends into the last hidden layer h, added to what the linear head left in dh [n][hid]
// (scratch: another [n][hid] buffer).
int aux_head_backward(Ctx* c, const bf16_t* h, int n, bool acc, bf16_t* dh, bf16_t* scratch) {
  if (c->XH <= 0) return PPO_OK;
  hipLaunchKernelGGL(k_aux_cols, dim3(cdiv((int64_t)n * 32, 256)), dim3(256), 0, c->stream, n, c->A_main, c->X, c->dhead, c->daux);
  LAUNCHCHK(c, "k_aux_cols");
  ARows dl2 = plain_arows(c->daux, HEAD_LD, n, HEAD_LD);
  ARows x2 = plain_arows(c->auxact, c->XH, n, c->XH);
  int rc = launch_wgrad(c, dl2, x2, c->X, c->XH, n, c->g + c->aux2W, c->g + c->aux2B, acc, "aux_wgrad.1", 2.0 * n * (c->XH + HEAD_LD));
  if (rc) return rc;
  Ep<MapRows, bf16_t, false, false, true> e2;
  e2.map = plain_map(c->XH, n); e2.out = c->dauxact; e2.bias = nullptr; e2.mask = c->auxact; e2.N = c->XH;
  rc = launch_gemm(c, dl2, n, c->aux2T, HEAD_LD, c->XH, HEAD_LD, e2, "aux_dgrad.1", 2.0 * n * (2.0 * c->XH + HEAD_LD));
  if (rc) return rc;
  ARows dl1 = plain_arows(c->dauxact, c->XH, n, c->XH);
  ARows x1 = plain_arows(h, c->hid, n, c->hid);
  rc = launch_wgrad(c, dl1, x1, c->XH, c->hid, n, c->g + c->aux1W, c->g + c->aux1B, acc, "aux_wgrad.0", 2.0 * n * ((double)c->hid + c->XH));
  if (rc) return rc;
  Ep<MapRows, bf16_t, false, false, true> e1;
  e1.map = plain_map(c->hid, n); e1.out = scratch; e1.bias = nullptr; e1.mask = h; e1.N = c->hid;
  rc = launch_gemm(c, dl1, n, c->aux1T, c->XH, c->hid, c->XH, e1, "aux_dgrad.0", 2.0 * n * (2.0 * c->hid + c->XH));
  if (rc) return rc;
  hipLaunchKernelGGL(k_add_bf16, dim3(cdiv((int64_t)n * c->hid / 8, 256)), dim3(256), 0, c->stream, (int64_t)n * c->hid / 8, dh, scratch);
  LAUNCHCHK(c, "k_add_bf16");
  return PPO_OK;
}

// Encoder of the feed-forward configurations: convolutions with fused bias + ReLU, the last one writing into the
// feature matrix, whose tail columns receive the proprioception.  `n` samples selected by device indices idx
// (NULL: samples first .. first + n - 1 of the buffer).
int encoder_forward_ff(Ctx* c, const int32_t* idx, int n, int64_t first) {
  const int V = c->V, nimg = n * V;
  bool proprio_done = false;
  if (idx) first = 0;
  const bf16_t* const proprio = c->proprio + first * c->P;
  {  // first convolution straight from the rollout buffer
    ImgAddr in; in.base = c->obs + first * c->img_elems * V; in.idx = idx; in.stride_b = c->img_elems * V; in.stride_v = c->img_elems; in.V = V;
    int Co = c->cC[1], Ho = c->cH[1], Wo = c->cW[1];
    int64_t M = (int64_t)nimg * Ho * Wo;
    ProfScope ps(c, "conv_fwd.0", 2.0 * (double)M * Co * 9 * c->cC[0], 2.0 * ((double)nimg * c->img_elems + (double)M * Co));
    constexpr int TPW = 4;
    const int grid = cdiv(M, 32 * 4 * TPW);
    Conv0Args ca;
    ca.in = in; ca.in.prepare(); ca.out = c->act[0]; ca.w = c->shadow + c->convW[0]; ca.bias = c->p + c->convB[0]; ca.zpage = c->zpage;
    ca.bits = c->nconv > 1 ? c->abits[0] : nullptr;
    ca.H = c->cH[0]; ca.W = c->cW[0]; ca.Ho = Ho; ca.Wo = Wo; ca.Cout = Co; ca.TR = 0; ca.NB = 0; ca.ntiles = 0;
    ca.tile_blocks = 0; ca.gather_blocks = 1; ca.pB = n; ca.P = c->P; ca.pcol0 = V * c->flat; ca.proprio = proprio; ca.feat = c->feat; ca.feat_ld = c->feat_ld;
    int trc = c->cC[0] == 1 ? launch_conv0_fwd_tile_t<1>(c, ca, nimg) : (c->cC[0] == 3 ? launch_conv0_fwd_tile_t<3>(c, ca, nimg) : 1);
    if (trc != PPO_OK && trc != 1) return trc;
    c->abits_ok[0] = trc == PPO_OK && c->nconv > 1;
    proprio_done = trc == PPO_OK;
    if (trc != PPO_OK) {  // shapes the LDS-ring kernel does not cover
      if (c->cC[0] == 1)
        hipLaunchKernelGGL((k_conv1_fwd<1, TPW>), dim3(grid), dim3(256), 0, c->stream, in, nimg, c->cH[0], c->cW[0], Ho, Wo, Co, c->shadow + c->convW[0], c->p + c->convB[0], c->act[0]);
      else
        hipLaunchKernelGGL((k_conv1_fwd<3, TPW>), dim3(grid), dim3(256), 0, c->stream, in, nimg, c->cH[0], c->cW[0], Ho, Wo, Co, c->shadow + c->convW[0], c->p + c->convB[0], c->act[0]);
      LAUNCHCHK(c, "k_conv1_fwd");
    }
  }
  for (int l = 1; l < c->nconv; ++l) {
    AConvFwd al;
    al.in = conv_out_addr(c, l - 1, c->act[l - 1], nullptr);
    al.H = c->cH[l]; al.W = c->cW[l]; al.Cin = c->cC[l]; al.lc = ilog2(al.Cin); al.Ho = c->cH[l + 1]; al.Wo = c->cW[l + 1];
    al.M = nimg * al.Ho * al.Wo; al.K = 9 * al.Cin;
    ImgAddr o = conv_out_addr(c, l, c->act[l], c->feat);
    Ep<MapRows, bf16_t, true, true, false> ep;
    ep.map.stride_b = o.stride_b; ep.map.stride_v = o.stride_v; ep.map.V = V; ep.map.HW = al.Ho * al.Wo; ep.map.C = c->cC[l + 1]; ep.map.M = al.M;
    ep.out = const_cast<bf16_t*>(o.base); ep.bias = c->p + c->convB[l]; ep.mask = nullptr; ep.N = c->cC[l + 1];
    double ab = 2.0 * ((double)nimg * al.H * al.W * al.Cin + (double)al.M * c->cC[l + 1] + (double)al.K * c->cC[l + 1]);
    const bool want_bits = l < c->nconv - 1;  // the last layer's mask is applied by the first linear layer's input gradient
    int rc = launch_conv_fwd_tile(c, al, o, c->cC[l + 1], c->shadow + c->convW[l], c->p + c->convB[l], nimg, "conv_fwd." + std::to_string(l), ab,
                                  want_bits ? c->abits[l] : nullptr);
    c->abits_ok[l] = want_bits && rc == PPO_OK;
    if (rc == PPO_OK + 1) rc = launch_gemm(c, al, al.M, c->shadow + c->convW[l], al.K, c->cC[l + 1], al.K, ep, "conv_fwd." + std::to_string(l), ab);
    if (rc) return rc;
  }
  if (!proprio_done) {  // (the first convolution's kernel copies the proprioception when it is the LDS-ring form)
    hipLaunchKernelGGL(k_gather_proprio, dim3(cdiv((int64_t)n * c->P, 256)), dim3(256), 0, c->stream, proprio, idx, n, c->P, c->feat, (int64_t)c->feat_ld, V * c->flat);
    LAUNCHCHK(c, "k_gather_proprio");
  }
  return PPO_OK;
}

// Hidden layers (bias, ReLU) on the trunk's input x [n][fin0] (row stride ldx), then the heads.
int trunk_forward(Ctx* c, const bf16_t* x, int64_t ldx, int n, bool with_head) {
  for (int l = 0; l < c->nfc; ++l) {
    ARows al = plain_arows(x, ldx, n, c->fin[l]);
    Ep<MapRows, bf16_t, true, true, false> ep;
    ep.map = plain_map(c->fout[l], n); ep.out = c->fcact[l]; ep.bias = c->p + c->fcB[l]; ep.mask = nullptr; ep.N = c->fout[l];
    double ab = 2.0 * ((double)n * c->fin[l] + (double)n * c->fout[l] + (double)c->fin[l] * c->fout[l]);
    int rc = launch_gemm(c, al, n, c->shadow + c->fcW[l], c->fin[l], c->fout[l], c->fin[l], ep, "fc_fwd." + std::to_string(l), ab);
    if (rc) return rc;
    x = c->fcact[l]; ldx = c->fout[l];
  }
  if (with_head) {
    ARows al = plain_arows(x, ldx, n, c->hid);
    Ep<MapRows, float, true, false, false> ep;
    ep.map = plain_map(HEAD_LD, n); ep.out = c->headout; ep.bias = c->p + c->headB; ep.mask = nullptr; ep.N = c->NH;
    int rc = launch_gemm(c, al, n, c->shadow + c->headW, c->hid, c->NH, c->hid, ep, "head_fwd", 2.0 * n * c->hid + 4.0 * n * c->NH);
    if (rc) return rc;
    rc = aux_head_forward(c, x, ldx, n);
    if (rc) return rc;
  }
  return PPO_OK;
}

int encoder_forward_generic(Ctx* c, const int32_t* idx, int n, int64_t first);

// Forward of `n` samples of a feed-forward network selected by device indices idx (NULL: samples first ..
// first + n - 1 of the buffer).
int forward_chunk(Ctx* c, const int32_t* idx, int n, bool with_head = true, int64_t first = 0) {
  const int rc = (c->ln || c->E > 0) ? encoder_forward_generic(c, idx, n, first) : encoder_forward_ff(c, idx, n, first);
  if (rc) return rc;
  return trunk_forward(c, c->feat, c->feat_ld, n, with_head);
}

// Backward of heads and hidden layers of a chunk whose forward activations are in the workspaces and whose
// head gradient is in dhead; xin [n][fin0] (row stride ldin) is the trunk's input.  Gradients land in c->g
// (overwritten, or added when `acc`); the gradient w.r.t. the trunk's input is left in gbuf[*cur_out] as
// [n][fin0], masked by xin > 0 when `mask_in` (xin is then a ReLU output).
int trunk_backward(Ctx* c, const bf16_t* xin, int64_t ldin, bool mask_in, int n, bool acc, bool with_head, int* cur_out) {
  int cur = 0;
  const bf16_t* hlast = c->fcact[c->nfc - 1];
  if (with_head) {  // heads (otherwise gbuf[0] already holds the gradient of the last hidden layer)
    ARows dl = plain_arows(c->dhead, HEAD_LD, n, HEAD_LD);
    ARows xl = plain_arows(hlast, c->hid, n, c->hid);
    int rc = launch_wgrad(c, dl, xl, c->NH, c->hid, n, c->g + c->headW, c->g + c->headB, acc, "head_wgrad", 2.0 * n * (c->hid + HEAD_LD));
    if (rc) return rc;
    Ep<MapRows, bf16_t, false, false, true> ep;
    ep.map = plain_map(c->hid, n); ep.out = c->gbuf[cur]; ep.bias = nullptr; ep.mask = hlast; ep.N = c->hid;
    rc = launch_gemm(c, dl, n, c->headT, HEAD_LD, c->hid, HEAD_LD, ep, "head_dgrad", 2.0 * n * (2.0 * c->hid + HEAD_LD));
    if (rc) return rc;
    rc = aux_head_backward(c, hlast, n, acc, c->gbuf[cur], c->gbuf[cur ^ 1]);
    if (rc) return rc;
  }
  for (int l = c->nfc - 1; l >= 0; --l) {
    const bf16_t* x = l ? c->fcact[l - 1] : xin;
    const int64_t ldx = l ? c->fin[l] : ldin;
    ARows dl = plain_arows(c->gbuf[cur], c->fout[l], n, c->fout[l]);
    ARows xl = plain_arows(x, ldx, n, c->fin[l]);
    int rc = launch_wgrad(c, dl, xl, c->fout[l], c->fin[l], n, c->g + c->fcW[l], c->g + c->fcB[l], acc, "fc_wgrad." + std::to_string(l),
                          2.0 * n * ((double)c->fin[l] + c->fout[l]) + 4.0 * (double)c->fin[l] * c->fout[l]);
    if (rc) return rc;
    const double ab = 2.0 * ((double)n * c->fout[l] + 2.0 * n * c->fin[l] + (double)c->fin[l] * c->fout[l]);
    if (l > 0 || mask_in) {
      Ep<MapRows, bf16_t, false, false, true> ep;
      ep.map = plain_map(c->fin[l], n); ep.out = c->gbuf[cur ^ 1]; ep.bias = nullptr; ep.mask = x; ep.N = c->fin[l];
      rc = launch_gemm(c, dl, n, c->fcT[l], c->fout[l], c->fin[l], c->fout[l], ep, "fc_dgrad." + std::to_string(l), ab);
    } else {  // the trunk's input is not a ReLU output (an embedding, an LSTM's h): nothing to mask
      Ep<MapRows, bf16_t, false, false, false> ep;
      ep.map = plain_map(c->fin[l], n); ep.out = c->gbuf[cur ^ 1]; ep.bias = nullptr; ep.mask = nullptr; ep.N = c->fin[l];
      rc = launch_gemm(c, dl, n, c->fcT[l], c->fout[l], c->fin[l], c->fout[l], ep, "fc_dgrad." + std::to_string(l), ab);
    }
    if (rc) return rc;
    cur ^= 1;
  }
  *cur_out = cur;
  return PPO_OK;
}

// Backward of the feed-forward configurations' convolutions from d(feat) in gbuf[cur] ([n][feat_ld], already masked
// by the last conv layer's ReLU).
int encoder_backward_ff(Ctx* c, const int32_t* idx, int n, bool acc, int cur) {
  const int V = c->V, nimg = n * V;
  for (int l = c->nconv - 1; l >= 1; --l) {
    const int Co = c->cC[l + 1], Ci = c->cC[l], Ho = c->cH[l + 1], Wo = c->cW[l + 1], H = c->cH[l], W = c->cW[l];
    ImgAddr dy = conv_out_addr(c, l, c->gbuf[cur], c->gbuf[cur]);
    ARows dl; dl.a = dy; dl.HW = Ho * Wo; dl.C = Co; dl.M = nimg * Ho * Wo; dl.K = Co; dl.plain = false;
    AConvFwd xl; xl.in = conv_out_addr(c, l - 1, c->act[l - 1], nullptr);
    xl.H = H; xl.W = W; xl.Cin = Ci; xl.lc = ilog2(Ci); xl.Ho = Ho; xl.Wo = Wo; xl.M = dl.M; xl.K = 9 * Ci;
    const double wab = 2.0 * ((double)dl.M * Co + (double)nimg * H * W * Ci) + 4.0 * 9.0 * Ci * Co;
    int rc = launch_conv_wgrad_tile(c, dy, xl, Co, nimg, c->g + c->convW[l], c->g + c->convB[l], acc, "conv_wgrad." + std::to_string(l), wab);
    if (rc == PPO_OK + 1)
      rc = launch_wgrad(c, dl, xl, Co, 9 * Ci, dl.M, c->g + c->convW[l], c->g + c->convB[l], acc, "conv_wgrad." + std::to_string(l), wab);
    if (rc) return rc;
    // transposed convolution over horizontal pixel pairs, both row parities in one launch (grid.z)
    AConvDgrad al; al.dy = dy; al.Ho = Ho; al.Wo = Wo; al.Cout = Co; al.lco = ilog2(Co); al.H = H; al.W = W; al.dy_imgs = nimg;
    al.w0 = c->wd[l][0]; al.w1 = c->wd[l][1];
    const int M0 = nimg * class_len(H, 0) * class_len(W, 0);  // the even-row parity sizes the grid
    ImgAddr xa = conv_out_addr(c, l - 1, c->act[l - 1], nullptr);
    Ep<MapDgrad, bf16_t, false, false, true> ep;
    ep.map.stride_b = xa.stride_b; ep.map.stride_v = xa.stride_v; ep.map.V = V; ep.map.H = H; ep.map.W = W; ep.map.Cin = Ci; ep.map.imgs = nimg;
    ep.out = c->gbuf[cur ^ 1]; ep.bias = nullptr; ep.mask = xa.base; ep.N = 2 * Ci;
    const bool dense_in = xa.stride_v == (int64_t)H * W * Ci && xa.stride_b == (int64_t)V * H * W * Ci;
    if (c->abits_ok[l - 1] && Ci % 32 == 0 && dense_in) ep.mbits = c->abits[l - 1];  // bit index = element offset of the dense activation
    const double pix = (double)nimg * H * W;
    const int N2 = 2 * Ci, BNf = N2 > 64 ? 128 : (N2 > 32 ? 64 : 32);
    const size_t wlds = (size_t)6 * Co * BNf * sizeof(bf16_t);  // both parities' packed weights, resident in LDS
    if (l == 1 && wlds <= 56 * 1024) {
      // fused with the first layer's weight gradient: its input gradient never leaves the chip
      ImgAddr in; in.base = c->obs; in.idx = idx; in.stride_b = c->img_elems * V; in.stride_v = c->img_elems; in.V = V;
      in.prepare(); al.prepare(); ep.map.prepare();
      const int K0 = 9 * c->cC[0], npair = Ci * (K0 + 1), tpp = cdiv(M0, 128);
      int grid = 2 * tpp < 512 ? 2 * tpp : 512;
      { const int erc = ensure_partial(c, (int64_t)grid * npair, 0); if (erc) return erc; }
      if ((int64_t)grid * npair > c->partial_elems) grid = (int)(c->partial_elems / npair);
      const double fflops = 2.0 * (double)nimg * Ho * Wo * 9.0 * Ci * Co + 2.0 * pix * Ci * (K0 + 1);
      // the ReLU mask is one bit per element when the forward kernel left its sign-bit words, else the stored activation
      const double fbytes = 2.0 * ((double)nimg * Ho * Wo * Co + (double)nimg * c->img_elems + 9.0 * Ci * Co) + (c->abits_ok[l - 1] ? pix * Ci / 8.0 : 2.0 * pix * Ci);
      int tgrid = 0;
      rc = launch_conv_dgrad_wgrad0_tile(c, dy, xa, c->abits_ok[l - 1] ? c->abits[l - 1] : nullptr, c->wtap[l], Co, Ci, H, W, Ho, Wo, in, c->cC[0], c->cH[0], c->cW[0], nimg,
                                         "conv_dgrad.1+wgrad.0", fflops, fbytes, &tgrid);
      if (rc == PPO_OK) grid = tgrid;
      else if (rc != PPO_OK + 1) return rc;
      else {
        rc = ensure_packed_dgrad_weights(c, l);
        if (rc) return rc;
        ProfScope ps(c, "conv_dgrad.1+wgrad.0", 2.0 * (double)nimg * Ho * Wo * 9.0 * Ci * Co + 2.0 * pix * Ci * (K0 + 1),
                     2.0 * ((double)nimg * Ho * Wo * Co + pix * Ci + (double)nimg * c->img_elems + 9.0 * Ci * Co));
#define LAUNCH_FUSED(BN_, WM_, WN_, CI0_)                                                                                                  \
        do {                                                                                                                                 \
          auto kfn = k_dgrad1_wgrad0<BN_, WM_, WN_, CI0_>;                                                                                   \
          HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)wlds));                            \
          hipLaunchKernelGGL(kfn, dim3(grid), dim3(256), wlds, c->stream, al, ep.map, xa.base, in, c->cH[0], c->cW[0], tpp, c->partial);      \
        } while (0)
        if (c->cC[0] == 1) {
          if (BNf == 128) LAUNCH_FUSED(128, 2, 2, 1); else if (BNf == 64) LAUNCH_FUSED(64, 2, 2, 1); else LAUNCH_FUSED(32, 4, 1, 1);
        } else {
          if (BNf == 128) LAUNCH_FUSED(128, 2, 2, 3); else if (BNf == 64) LAUNCH_FUSED(64, 2, 2, 3); else LAUNCH_FUSED(32, 4, 1, 3);
        }
#undef LAUNCH_FUSED
        LAUNCHCHK(c, "k_dgrad1_wgrad0");
      }
      defer_reduce(c, 2, grid, npair, Ci, K0, c->g + c->convW[0], c->g + c->convB[0], acc, false, 0, nullptr);
      return flush_reduces(c);
    }
    double ab = 2.0 * ((double)nimg * Ho * Wo * Co + pix * Ci + 9.0 * Ci * Co) + (c->abits_ok[l - 1] && (Co == 64 || ep.mbits) ? pix * Ci / 8.0 : 2.0 * pix * Ci);
    const double dflops = 2.0 * (double)nimg * Ho * Wo * 9.0 * Ci * Co;
    rc = launch_conv_dgrad_tile(c, dy, xa, c->abits_ok[l - 1] ? c->abits[l - 1] : nullptr, c->gbuf[cur ^ 1], c->wtap[l], Co, Ci, H, W, Ho, Wo, nimg, "conv_dgrad." + std::to_string(l), dflops, ab);
    if (rc == PPO_OK + 1) {
      rc = ensure_packed_dgrad_weights(c, l);
      if (rc) return rc;
      rc = launch_gemm(c, al, M0, nullptr, 0, 2 * Ci, 4 * Co, ep, "conv_dgrad." + std::to_string(l), ab, 2, dflops);
    }
    if (rc) return rc;
    cur ^= 1;
  }
  {  // first convolution: weight and bias gradient only
    ImgAddr in; in.base = c->obs; in.idx = idx; in.stride_b = c->img_elems * V; in.stride_v = c->img_elems; in.V = V;
    const int Co = c->cC[1], Ho = c->cH[1], Wo = c->cW[1], K = 9 * c->cC[0];
    int64_t M = (int64_t)nimg * Ho * Wo;
    const int npair = Co * (K + 1);
    { const int erc = ensure_partial(c, (int64_t)2048 * npair, 0); if (erc) return erc; }
    int64_t max_blocks = c->partial_elems / npair;
    if (max_blocks > 2048) max_blocks = 2048;
    int64_t ppb = (M + max_blocks - 1) / max_blocks;
    ppb = (ppb + 63) / 64 * 64;
    int nblk = cdiv(M, ppb);
    ProfScope ps(c, "conv_wgrad.0", 2.0 * (double)M * Co * (K + 1), 2.0 * ((double)M * Co + (double)nimg * c->img_elems));
    if (c->cC[0] == 1)
      hipLaunchKernelGGL((k_conv1_wgrad<1>), dim3(nblk), dim3(256), 0, c->stream, in, nimg, c->cH[0], c->cW[0], Ho, Wo, Co, c->gbuf[cur], (int)ppb, c->partial);
    else
      hipLaunchKernelGGL((k_conv1_wgrad<3>), dim3(nblk), dim3(256), 0, c->stream, in, nimg, c->cH[0], c->cW[0], Ho, Wo, Co, c->gbuf[cur], (int)ppb, c->partial);
    LAUNCHCHK(c, "k_conv1_wgrad");
    defer_reduce(c, 2, nblk, npair, Co, K, c->g + c->convW[0], c->g + c->convB[0], acc, false, 0, nullptr);
  }
  return flush_reduces(c);
}

int encoder_backward_generic(Ctx* c, const int32_t* idx, int n, bool acc, int cur);
int encoder_forward_generic(Ctx* c, const int32_t* idx, int n, int64_t first);

// Backward of a feed-forward chunk whose forward activations are in the workspaces and whose head gradient is
// in dhead.  Gradients land in c->g (overwritten, or added when `acc`).
int backward_chunk(Ctx* c, const int32_t* idx, int n, bool acc, bool with_head = true) {
  int cur = 0;
  const bool generic = c->ln || c->E > 0;
  int rc = trunk_backward(c, c->feat, c->feat_ld, c->E == 0, n, acc, with_head, &cur);
  if (rc) return rc;
  return generic ? encoder_backward_generic(c, idx, n, acc, cur) : encoder_backward_ff(c, idx, n, acc, cur);
}

// ---------------------------------------------------------------- encoder with layer normalisation and / or embedding
// Every convolution through the implicit-GEMM kernels without the fused ReLU; with layer_norm the convolution
// output is stored (pre), normalised per image and rectified by k_ln_fwd; without it the ReLU stays in the
// convolution's epilogue.  The last layer's activation goes into the feature matrix, or (embed_dim > 0) into a
// buffer of its own that the embedding GEMM reads, view by view.
static ImgAddrW as_w(const ImgAddr& a) { ImgAddrW w; w.base = const_cast<bf16_t*>(a.base); w.stride_b = a.stride_b; w.stride_v = a.stride_v; w.V = a.V; return w; }
static ImgAddr contiguous_imgs(const bf16_t* base, int64_t e, int V) { ImgAddr a; a.base = base; a.idx = nullptr; a.stride_b = e * V; a.stride_v = e; a.V = V; return a; }
// where the output activation of conv layer l lives for a chunk
static ImgAddr act_addr(Ctx* c, int l) {
  const int64_t e = (int64_t)c->cC[l + 1] * c->cH[l + 1] * c->cW[l + 1];
  if (l == c->nconv - 1 && c->E == 0) { ImgAddr a; a.base = c->feat; a.idx = nullptr; a.stride_b = c->feat_ld; a.stride_v = c->flat; a.V = c->V; return a; }
  return contiguous_imgs(c->act[l], e, c->V);
}

int encoder_forward_generic(Ctx* c, const int32_t* idx, int n, int64_t first) {
  const int V = c->V, nimg = n * V;
  if (idx) first = 0;
  for (int l = 0; l < c->nconv; ++l) {
    const int Co = c->cC[l + 1], Ho = c->cH[l + 1], Wo = c->cW[l + 1], Ci = c->cC[l];
    const int64_t e = (int64_t)Co * Ho * Wo, M = (int64_t)nimg * Ho * Wo;
    const ImgAddr oa = act_addr(c, l);
    const ImgAddr conv_to = c->ln ? contiguous_imgs(c->pre[l], e, V) : oa;
    const std::string name = "conv_fwd." + std::to_string(l);
    if (l == 0) {
      ImgAddr in; in.base = c->obs + first * c->img_elems * V; in.idx = idx; in.stride_b = c->img_elems * V; in.stride_v = c->img_elems; in.V = V;
      in.prepare();
      if (conv_to.stride_v != e || conv_to.stride_b != e * V) return fail(c, PPO_ESHAPE, "the first convolution needs a contiguous output (n_conv >= 2 or an embedding)");
      ProfScope ps(c, name, 2.0 * (double)M * Co * 9 * Ci, 2.0 * ((double)nimg * c->img_elems + (double)M * Co));
      constexpr int TPW = 4;
      const int grid = cdiv(M, 32 * 4 * TPW);
      bf16_t* out = const_cast<bf16_t*>(conv_to.base);
      const bf16_t* w = c->shadow + c->convW[0];
      const float* b = c->p + c->convB[0];
#define LAUNCH_C1(CIN_, RELU_) hipLaunchKernelGGL((k_conv1_fwd<CIN_, TPW, RELU_>), dim3(grid), dim3(256), 0, c->stream, in, nimg, c->cH[0], c->cW[0], Ho, Wo, Co, w, b, out)
      if (Ci == 1) { if (c->ln) LAUNCH_C1(1, false); else LAUNCH_C1(1, true); }
      else { if (c->ln) LAUNCH_C1(3, false); else LAUNCH_C1(3, true); }
#undef LAUNCH_C1
      LAUNCHCHK(c, "k_conv1_fwd");
    } else {
      AConvFwd al;
      al.in = act_addr(c, l - 1);
      al.H = c->cH[l]; al.W = c->cW[l]; al.Cin = Ci; al.lc = ilog2(Ci); al.Ho = Ho; al.Wo = Wo; al.M = (int)M; al.K = 9 * Ci;
      const double ab = 2.0 * ((double)nimg * al.H * al.W * Ci + (double)M * Co + (double)al.K * Co);
      int rc;
      if (c->ln) {
        Ep<MapRows, bf16_t, true, false, false> ep;
        ep.map.stride_b = conv_to.stride_b; ep.map.stride_v = conv_to.stride_v; ep.map.V = V; ep.map.HW = Ho * Wo; ep.map.C = Co; ep.map.M = (int)M;
        ep.out = const_cast<bf16_t*>(conv_to.base); ep.bias = c->p + c->convB[l]; ep.mask = nullptr; ep.N = Co;
        rc = launch_gemm(c, al, (int)M, c->shadow + c->convW[l], al.K, Co, al.K, ep, name, ab);
      } else {
        Ep<MapRows, bf16_t, true, true, false> ep;
        ep.map.stride_b = conv_to.stride_b; ep.map.stride_v = conv_to.stride_v; ep.map.V = V; ep.map.HW = Ho * Wo; ep.map.C = Co; ep.map.M = (int)M;
        ep.out = const_cast<bf16_t*>(conv_to.base); ep.bias = c->p + c->convB[l]; ep.mask = nullptr; ep.N = Co;
        rc = launch_gemm(c, al, (int)M, c->shadow + c->convW[l], al.K, Co, al.K, ep, name, ab);
      }
      if (rc) return rc;
    }
    c->abits_ok[l] = false;
    if (c->ln) {
      ProfScope ps(c, "layer_norm_fwd", 8.0 * (double)nimg * e, 4.0 * (double)nimg * e);
      // an image that fits one block's registers is read once
      const int64_t pch = cdiv(e / 8, LN_RTHREADS);  // 16-byte chunks per thread
      if (pch <= 2 && Co <= 512) hipLaunchKernelGGL(k_ln_fwd_reg<2>, dim3(nimg), dim3(LN_RTHREADS), 0, c->stream, c->pre[l], (int)e, Co, c->p + c->lnG[l], c->p + c->lnB[l], as_w(oa), c->lnstat[l]);
      else if (pch <= 5 && Co <= 512) hipLaunchKernelGGL(k_ln_fwd_reg<5>, dim3(nimg), dim3(LN_RTHREADS), 0, c->stream, c->pre[l], (int)e, Co, c->p + c->lnG[l], c->p + c->lnB[l], as_w(oa), c->lnstat[l]);
      else if (pch <= 10 && Co <= 512) hipLaunchKernelGGL(k_ln_fwd_reg<10>, dim3(nimg), dim3(LN_RTHREADS), 0, c->stream, c->pre[l], (int)e, Co, c->p + c->lnG[l], c->p + c->lnB[l], as_w(oa), c->lnstat[l]);
      else
      hipLaunchKernelGGL(k_ln_fwd, dim3(nimg), dim3(LN_THREADS), 0, c->stream, c->pre[l], (int)e, Co, c->p + c->lnG[l], c->p + c->lnB[l], as_w(oa), c->lnstat[l]);
      LAUNCHCHK(c, "k_ln_fwd");
    }
  }
  if (c->E > 0) {  // embedding of each view's flattened features: a linear layer, no activation
    for (int v = 0; v < V; ++v) {
      ARows al = plain_arows(c->act[c->nconv - 1] + (int64_t)v * c->flat, (int64_t)V * c->flat, n, c->flat);
      Ep<MapRows, bf16_t, true, false, false> ep;
      ep.map = plain_map(c->feat_ld, n); ep.out = c->feat + (int64_t)v * c->E; ep.bias = c->p + c->embB; ep.mask = nullptr; ep.N = c->E;
      const int rc = launch_gemm(c, al, n, c->shadow + c->embW, c->flat, c->E, c->flat, ep, "embed_fwd", 2.0 * ((double)n * c->flat + (double)n * c->E + (double)c->flat * c->E));
      if (rc) return rc;
    }
  }
  hipLaunchKernelGGL(k_gather_proprio, dim3(cdiv((int64_t)n * c->P, 256)), dim3(256), 0, c->stream, c->proprio + first * c->P, idx, n, c->P, c->feat,
                     (int64_t)c->feat_ld, V * c->enc);
  LAUNCHCHK(c, "k_gather_proprio");
  return PPO_OK;
}

// Its backward from d(features) in `dfeat` (row stride ld_df; with an embedding its columns [v*E, (v+1)*E) are the
// gradient of view v's embedding, without one the masked gradient of the last convolution's activation).
int encoder_backward_seq(Ctx* c, const int32_t* idx, int n, bool acc, const bf16_t* dfeat, int64_t ld_df, int cur) {
  const int V = c->V, nimg = n * V, L = c->nconv;
  // gradient w.r.t. the last convolution's activation, masked by its ReLU
  ImgAddr dy;
  if (c->E > 0) {
    bf16_t* dst = c->gbuf[cur ^ 1];
    for (int v = 0; v < V; ++v) {
      ARows dl = plain_arows(dfeat + (int64_t)v * c->E, ld_df, n, c->E);
      ARows xl = plain_arows(c->act[L - 1] + (int64_t)v * c->flat, (int64_t)V * c->flat, n, c->flat);
      int rc = launch_wgrad(c, dl, xl, c->E, c->flat, n, c->g + c->embW, c->g + c->embB, acc || v > 0, "embed_wgrad", 2.0 * n * ((double)c->flat + c->E));
      if (rc) return rc;
      Ep<MapRows, bf16_t, false, false, true> ep;
      ep.map = plain_map((int64_t)V * c->flat, n); ep.out = dst + (int64_t)v * c->flat; ep.bias = nullptr; ep.mask = c->act[L - 1] + (int64_t)v * c->flat; ep.N = c->flat;
      rc = launch_gemm(c, dl, n, c->embT, c->E, c->flat, c->E, ep, "embed_dgrad", 2.0 * n * (2.0 * c->flat + c->E));
      if (rc) return rc;
    }
    cur ^= 1;
    dy = contiguous_imgs(c->gbuf[cur], c->flat, V);
  } else {
    if (c->nl > 0 && !c->ln) {  // the LSTM's GEMM left this gradient unmasked, and no layer-norm backward will mask it
      hipLaunchKernelGGL(k_mask_rows, dim3(cdiv((int64_t)n * (V * c->flat / 8), 256)), dim3(256), 0, c->stream, (int64_t)n, V * c->flat, const_cast<bf16_t*>(dfeat), ld_df,
                         c->feat, (int64_t)c->feat_ld);
      LAUNCHCHK(c, "k_mask_rows");
    }
    dy.base = dfeat; dy.idx = nullptr; dy.stride_b = ld_df; dy.stride_v = c->flat; dy.V = V;
  }
  for (int l = L - 1; l >= 0; --l) {
    const int Co = c->cC[l + 1], Ci = c->cC[l], Ho = c->cH[l + 1], Wo = c->cW[l + 1], H = c->cH[l], W = c->cW[l];
    const int64_t e = (int64_t)Co * Ho * Wo;
    ImgAddr dconv = dy;  // gradient w.r.t. the convolution's output
    if (c->ln) {
      int grid = nimg < 1024 ? nimg : 1024;
      { const int erc = ensure_partial(c, (int64_t)grid * 2 * Co, 0); if (erc) return erc; }
      if ((int64_t)grid * 2 * Co > c->partial_elems) grid = (int)(c->partial_elems / (2 * Co));
      if (grid < 1) return fail(c, PPO_ENOMEM, "weight-gradient workspace too small for the layer-norm gradients");
      {
        ProfScope ps(c, "layer_norm_bwd", 14.0 * (double)nimg * e, 6.0 * (double)nimg * e);
        dy.prepare();
        hipLaunchKernelGGL(k_ln_bwd, dim3(grid), dim3(LN_THREADS), 0, c->stream, dy, c->pre[l], c->lnstat[l], nimg, (int)e, Co, c->p + c->lnG[l], c->p + c->lnB[l], c->dpre, c->partial);
        LAUNCHCHK(c, "k_ln_bwd");
      }
      defer_reduce(c, 0, grid, 2 * Co, 0, 0, c->g + c->lnG[l], nullptr, acc, false, 0, nullptr);  // gain and shift gradients are adjacent
      dconv = contiguous_imgs(c->dpre, e, V);
    }
    if (l == 0) {
      ImgAddr in; in.base = c->obs; in.idx = idx; in.stride_b = c->img_elems * V; in.stride_v = c->img_elems; in.V = V;
      if (dconv.stride_v != e || dconv.stride_b != e * V) return fail(c, PPO_ESHAPE, "the first convolution's gradient needs a contiguous layout");
      const int K = 9 * Ci;
      int64_t M = (int64_t)nimg * Ho * Wo;
      const int npair = Co * (K + 1);
      { const int erc = ensure_partial(c, (int64_t)2048 * npair, 0); if (erc) return erc; }
      int64_t max_blocks = c->partial_elems / npair;
      if (max_blocks > 2048) max_blocks = 2048;
      if (max_blocks < 1) return fail(c, PPO_ENOMEM, "weight-gradient workspace too small for the first convolution");
      int64_t ppb = (M + max_blocks - 1) / max_blocks;
      ppb = (ppb + 63) / 64 * 64;
      const int nblk = cdiv(M, ppb);
      ProfScope ps(c, "conv_wgrad.0", 2.0 * (double)M * Co * (K + 1), 2.0 * ((double)M * Co + (double)nimg * c->img_elems));
      if (Ci == 1) hipLaunchKernelGGL((k_conv1_wgrad<1>), dim3(nblk), dim3(256), 0, c->stream, in, nimg, H, W, Ho, Wo, Co, dconv.base, (int)ppb, c->partial);
      else hipLaunchKernelGGL((k_conv1_wgrad<3>), dim3(nblk), dim3(256), 0, c->stream, in, nimg, H, W, Ho, Wo, Co, dconv.base, (int)ppb, c->partial);
      LAUNCHCHK(c, "k_conv1_wgrad");
      defer_reduce(c, 2, nblk, npair, Co, K, c->g + c->convW[0], c->g + c->convB[0], acc, false, 0, nullptr);
      break;
    }
    ARows dl; dl.a = dconv; dl.HW = Ho * Wo; dl.C = Co; dl.M = nimg * Ho * Wo; dl.K = Co; dl.plain = false;
    AConvFwd xl; xl.in = act_addr(c, l - 1);
    xl.H = H; xl.W = W; xl.Cin = Ci; xl.lc = ilog2(Ci); xl.Ho = Ho; xl.Wo = Wo; xl.M = dl.M; xl.K = 9 * Ci;
    const double wab = 2.0 * ((double)dl.M * Co + (double)nimg * H * W * Ci) + 4.0 * 9.0 * Ci * Co;
    int rc = launch_wgrad(c, dl, xl, Co, 9 * Ci, dl.M, c->g + c->convW[l], c->g + c->convB[l], acc, "conv_wgrad." + std::to_string(l), wab);
    if (rc) return rc;
    AConvDgrad al; al.dy = dconv; al.Ho = Ho; al.Wo = Wo; al.Cout = Co; al.lco = ilog2(Co); al.H = H; al.W = W; al.dy_imgs = nimg;
    rc = ensure_packed_dgrad_weights(c, l);
    if (rc) return rc;
    al.w0 = c->wd[l][0]; al.w1 = c->wd[l][1];
    const int M0 = nimg * class_len(H, 0) * class_len(W, 0);
    const ImgAddr xa = act_addr(c, l - 1);
    Ep<MapDgrad, bf16_t, false, false, true> ep;
    ep.map.stride_b = xa.stride_b; ep.map.stride_v = xa.stride_v; ep.map.V = V; ep.map.H = H; ep.map.W = W; ep.map.Cin = Ci; ep.map.imgs = nimg;
    ep.out = c->gbuf[cur ^ 1]; ep.bias = nullptr; ep.mask = xa.base; ep.N = 2 * Ci;
    const bool dense_in = xa.stride_v == (int64_t)H * W * Ci && xa.stride_b == (int64_t)V * H * W * Ci;
    if (c->abits_ok[l - 1] && Ci % 32 == 0 && dense_in) ep.mbits = c->abits[l - 1];  // bit index = element offset of the dense activation
    const double pix = (double)nimg * H * W;
    rc = launch_gemm(c, al, M0, nullptr, 0, 2 * Ci, 4 * Co, ep, "conv_dgrad." + std::to_string(l),
                     2.0 * ((double)nimg * Ho * Wo * Co + 2.0 * pix * Ci + 9.0 * Ci * Co), 2, 2.0 * (double)nimg * Ho * Wo * 9.0 * Ci * Co);
    if (rc) return rc;
    cur ^= 1;
    dy = contiguous_imgs(c->gbuf[cur], (int64_t)Ci * H * W, V);
  }
  return flush_reduces(c);
}
int encoder_backward_generic(Ctx* c, const int32_t* idx, int n, bool acc, int cur) {
  return encoder_backward_seq(c, idx, n, acc, c->gbuf[cur], c->fin[0], cur);
}

// ---------------------------------------------------------------- recurrent core
// Forward of a chunk of `ne` whole environments (device list env) x T steps, rows time-major.  Encoder on all
// ne*T rows at once, then per LSTM layer and step one GEMM (the operand row [x_t, h_enter] against the layer's
// [W_ih, W_hh]) and one cell kernel, then hidden layers and heads on all rows.
int forward_seq_chunk(Ctx* c, const int32_t* env, int ne, bool with_head) {
  const int T = c->T, n = ne * T, H = c->H;
  hipLaunchKernelGGL(k_seq_index, dim3(cdiv(n, 256)), dim3(256), 0, c->stream, env, ne, T, c->N, c->seqidx);
  LAUNCHCHK(c, "k_seq_index");
  int rc = (c->ln || c->E > 0) ? encoder_forward_generic(c, c->seqidx, n, 0) : encoder_forward_ff(c, c->seqidx, n, 0);
  if (rc) return rc;
  for (int l = 0; l < c->nl; ++l) {
    const int K = c->lin[l] + H;
    hipLaunchKernelGGL(k_lstm_init, dim3(cdiv(ne * H, 256)), dim3(256), 0, c->stream, env, ne, H, c->h0 + (int64_t)l * c->N * H, c->c0 + (int64_t)l * c->N * H,
                       c->xh[l], (int64_t)K, c->lin[l], c->c_enter[l]);
    LAUNCHCHK(c, "k_lstm_init");
    const bool top = l == c->nl - 1;
    bf16_t* outm = top ? c->htop : c->xh[l + 1];
    const int64_t ld_out = top ? H : c->lin[l + 1] + H;
    for (int t = 0; t < T; ++t) {
      const int64_t r0 = (int64_t)t * ne;
      ARows al = plain_arows(c->xh[l] + r0 * K, K, ne, K);
      Ep<MapRows, float, true, false, false> ep;
      ep.map = plain_map(4 * H, ne); ep.out = c->lstm_pre; ep.bias = c->p + c->lstmB[l]; ep.mask = nullptr; ep.N = 4 * H;
      rc = launch_gemm(c, al, ne, c->shadow + c->lstmW[l], K, 4 * H, K, ep, "lstm_fwd." + std::to_string(l), 2.0 * ((double)ne * K + (double)K * 4 * H) + 16.0 * ne * H);
      if (rc) return rc;
      ProfScope ps(c, "lstm_cell_fwd", 30.0 * ne * H, (double)ne * H * (16.0 + 16.0 + 8.0 + 4.0));
      const bool last = t == T - 1;
      hipLaunchKernelGGL(k_lstm_cell_fwd, dim3(cdiv(ne * H, 256)), dim3(256), 0, c->stream, ne, H, c->lstm_pre, c->c_enter[l] + r0 * H, c->done, c->seqidx + r0,
                         c->gates[l] + r0 * 4 * H, outm + r0 * ld_out, ld_out, last ? nullptr : c->xh[l] + (r0 + ne) * K + c->lin[l], (int64_t)K,
                         last ? nullptr : c->c_enter[l] + (r0 + ne) * H);
      LAUNCHCHK(c, "k_lstm_cell_fwd");
    }
  }
  return trunk_forward(c, c->nl > 0 ? c->htop : c->feat, c->nl > 0 ? (int64_t)H : c->feat_ld, n, with_head);
}

// Its backward: heads and hidden layers on all rows, then back-propagation through time per LSTM layer (top
// first): per step the cell's backward kernel and one GEMM that turns the gate gradients into the gradient of
// the operand row [x_t, h_enter] - its h half is what step t-1 receives -; the layer's weight gradient is one
// contraction over all rows afterwards.  Then the encoder's backward on all rows.
int backward_seq_chunk(Ctx* c, int ne, bool acc, bool with_head) {
  const int T = c->T, n = ne * T, H = c->H;
  int cur = 0;
  int rc = trunk_backward(c, c->htop, H, false, n, acc, with_head, &cur);
  if (rc) return rc;
  const bf16_t* dabove = c->gbuf[cur];
  int64_t ld_above = H;
  for (int l = c->nl - 1; l >= 0; --l) {
    const int K = c->lin[l] + H;
    for (int t = T - 1; t >= 0; --t) {
      const int64_t r0 = (int64_t)t * ne;
      const bool last = t == T - 1;
      {
        ProfScope ps(c, "lstm_cell_bwd", 40.0 * ne * H, (double)ne * H * (16.0 + 4.0 + 4.0 + 8.0 + 8.0));
        hipLaunchKernelGGL(k_lstm_cell_bwd, dim3(cdiv(ne * H, 256)), dim3(256), 0, c->stream, ne, H, c->gates[l] + r0 * 4 * H, c->c_enter[l] + r0 * H, c->done,
                           c->seqidx + r0, dabove + r0 * ld_above, ld_above, last ? nullptr : c->dxh[l] + (r0 + ne) * K + c->lin[l], (int64_t)K, c->dc_carry,
                           last ? 1 : 0, c->da + r0 * 4 * H);
        LAUNCHCHK(c, "k_lstm_cell_bwd");
      }
      ARows dl = plain_arows(c->da + r0 * 4 * H, 4 * H, ne, 4 * H);
      Ep<MapRows, bf16_t, false, false, false> ep;
      ep.map = plain_map(K, ne); ep.out = c->dxh[l] + r0 * K; ep.bias = nullptr; ep.mask = nullptr; ep.N = K;
      rc = launch_gemm(c, dl, ne, c->lstmWT[l], 4 * H, K, 4 * H, ep, "lstm_dgrad." + std::to_string(l), 2.0 * ((double)ne * 4 * H + (double)ne * K + (double)K * 4 * H));
      if (rc) return rc;
    }
    ARows dl = plain_arows(c->da, 4 * H, n, 4 * H);
    ARows xl = plain_arows(c->xh[l], K, n, K);
    rc = launch_wgrad(c, dl, xl, 4 * H, K, n, c->g + c->lstmW[l], c->g + c->lstmB[l], acc, "lstm_wgrad." + std::to_string(l), 2.0 * n * ((double)K + 4 * H) + 4.0 * (double)K * 4 * H);
    if (rc) return rc;
    dabove = c->dxh[l]; ld_above = K;   // the x half of this layer's operand gradient is the layer below's dh
  }
  return encoder_backward_seq(c, c->seqidx, n, acc, c->dxh[0], c->lin[0] + H, cur);
}

// The permutations of epochs epoch0 .. epoch0 + count - 1 (count <= PERM_BATCH) of (seed, update) into the slots
// 0 .. count - 1 of c->perm ([PERM_BATCH][S]): five launches whatever the count.
int gen_permutations(Ctx* c, uint64_t seed, uint64_t update, uint64_t epoch0, int count) {
  PermStreams ps;
  for (int e = 0; e < PERM_BATCH; ++e) ps.s[e] = perm_stream(seed, update, epoch0 + (uint64_t)(e < count ? e : 0));
  const int S = c->PU, g = cdiv(S, 256), nb = c->nb;  // the units a minibatch is made of: samples, or whole environments
  ProfScope pscope(c, "permutation", 0.0, 4.0 * S * count);
  hipLaunchKernelGGL(k_fill_i32, dim3(cdiv((int64_t)count * 2 * nb, 256)), dim3(256), 0, c->stream, c->phist, (int64_t)count * 2 * nb, 0);  // hist + cursor
  hipLaunchKernelGGL(k_perm_hist, dim3(g, count), dim3(256), 0, c->stream, ps, S, c->shift, nb, c->phist);
  hipLaunchKernelGGL(k_perm_scan, dim3(1, count), dim3(1024), 0, c->stream, c->phist, c->pstart, nb);
  hipLaunchKernelGGL(k_perm_scatter, dim3(g, count), dim3(256), 0, c->stream, ps, S, c->shift, nb, c->pstart, c->phist, c->ptmp);
  hipLaunchKernelGGL(k_perm_rank, dim3(g, count), dim3(256), 0, c->stream, ps, S, c->shift, nb, c->pstart, c->phist, c->ptmp, c->perm);
  LAUNCHCHK(c, "permutation kernels");
  return PPO_OK;
}
int gen_permutation(Ctx* c, uint64_t seed, uint64_t update, uint64_t epoch) { return gen_permutations(c, seed, update, epoch, 1); }

// Output layer forward, loss and output layer backward of a chunk in one kernel (head_loss.hip.h);
// returns 1 when the width of the last hidden layer or the workspaces do not allow it.
template <int HID>
int launch_head_loss_t(Ctx* c, const LossData& L, int n, bool acc, bool distill, float* sp, float* dp) {
  typedef HeadLossShape<HID> S;
  const int nblk = cdiv(n, 64);
  { const int erc = ensure_partial(c, (int64_t)nblk * c->NH * HID, (int64_t)nblk * c->NH); if (erc) return erc; }
  if ((int64_t)nblk * c->NH * HID > c->partial_elems || (int64_t)nblk * c->NH > c->bias_partial_elems) return 1;
  HeadLossArgs a;
  a.h = c->fcact[c->nfc - 1]; a.w = c->shadow + c->headW; a.wt = c->headT; a.bias = c->p + c->headB; a.dh = c->gbuf[0];
  a.wpart = c->partial; a.bpart = c->bias_partial; a.stat_part = sp; a.dls_part = dp; a.n = n; a.NH = c->NH;
  {
    ProfScope ps(c, "head+loss", 6.0 * n * (double)HID * HEAD_LD, (double)n * (4.0 * HID + 4.0 * c->A + 20.0));
    static uint64_t attr_devs[2] = {0, 0};  // bit d: set on device d
    if (distill) {
      auto kfn = k_head_loss<HID, true>;
      if (!((attr_devs[1] >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS_BYTES)); attr_devs[1] |= 1ull << c->dev; }
      hipLaunchKernelGGL(kfn, dim3(nblk), dim3(256), S::LDS_BYTES, c->stream, a, L);
    } else {
      auto kfn = k_head_loss<HID, false>;
      if (!((attr_devs[0] >> c->dev) & 1)) { HIPCHK(c, hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, S::LDS_BYTES)); attr_devs[0] |= 1ull << c->dev; }
      hipLaunchKernelGGL(kfn, dim3(nblk), dim3(256), S::LDS_BYTES, c->stream, a, L);
    }
    LAUNCHCHK(c, "k_head_loss");
  }
  defer_reduce(c, 0, nblk, (int64_t)c->NH * HID, 0, 0, c->g + c->headW, nullptr, acc, true, c->NH, c->g + c->headB);
  return PPO_OK;
}
int launch_head_loss(Ctx* c, const LossData& L, int n, bool acc, bool distill, float* sp, float* dp) {
  if (c->NH > HEAD_LD || c->nfc < 1) return 1;
  switch (c->hid) {
    case 32: return launch_head_loss_t<32>(c, L, n, acc, distill, sp, dp);
    case 64: return launch_head_loss_t<64>(c, L, n, acc, distill, sp, dp);
    case 128: return launch_head_loss_t<128>(c, L, n, acc, distill, sp, dp);
    default: return 1;
  }
}
bool head_loss_covers(const Ctx* c) { return c->XH == 0 && c->NH <= HEAD_LD && c->nfc >= 1 && (c->hid == 32 || c->hid == 64 || c->hid == 128); }

int run_update(Ctx* c, const ppo_hparams* hp, ppo_mb_stats* host_stats, bool distill) {
  // a minibatch is Bu units of L rows each: samples (L = 1), or whole environments of T steps (recurrent nets)
  const bool recurrent = c->nl > 0;
  const int L = recurrent ? c->T : 1, Bu = c->PU / hp->minibatches, CU = recurrent ? c->CHe : c->CH;
  const int B = Bu * L;
  const int steps = hp->epochs * hp->minibatches;
  const int blocks_per_chunk = cdiv(CU * L, LOSS_BLOCK);
  int k = 0;
  const bool adaptive = !distill && hp->desired_kl > 0.f;  // the learning rate lives on the device and follows approx_kl
  if (!distill && hp->norm_adv) {
    ProfScope ps(c, "adv_normalize", 0.0, 12.0 * c->S);
    int per = cdiv(c->S, ADVN_BLOCKS);
    if (per < 4096) per = 4096;  // a block is worth launching for a few samples per thread
    const int nblk = cdiv(c->S, per);
    hipLaunchKernelGGL(k_adv_stats, dim3(nblk), dim3(1024), 0, c->stream, c->S, per, c->adv, c->advn_part);
    hipLaunchKernelGGL(k_adv_apply, dim3(nblk), dim3(1024), 0, c->stream, c->S, per, nblk, c->adv, c->advn_part, c->adv_n);
    LAUNCHCHK(c, "advantage normalisation");
  }
  for (int e = 0; e < hp->epochs; ++e) {
    int rc = PPO_OK;
    // the permutations of the next PERM_BATCH epochs in one set of launches (those of the last set are no longer read)
    if (e % PERM_BATCH == 0) rc = gen_permutations(c, hp->seed, (uint64_t)c->update_idx, (uint64_t)e, hp->epochs - e < PERM_BATCH ? hp->epochs - e : PERM_BATCH);
    if (rc) return rc;
    for (int mb = 0; mb < hp->minibatches; ++mb, ++k) {
      const int32_t* units = c->perm + (int64_t)(e % PERM_BATCH) * c->PU + (int64_t)mb * Bu;
      int nblocks = 0;
      for (int c0 = 0, ci = 0; c0 < Bu; c0 += CU, ++ci) {
        const int nu = (Bu - c0 < CU) ? Bu - c0 : CU, n = nu * L;
        const bool fused_head = head_loss_covers(c);
        // the rollout samples of the chunk's rows: the permutation's entries themselves, or the index list that
        // forward_seq_chunk builds from the chunk's environments
        const int32_t* rows = recurrent ? c->seqidx : units + c0;
        rc = recurrent ? forward_seq_chunk(c, units + c0, nu, !fused_head) : forward_chunk(c, rows, n, !fused_head);
        if (rc) return rc;
        float* sp = c->stat_part + (int64_t)ci * blocks_per_chunk * LOSS_NSTAT;
        float* dp = c->dls_part + (int64_t)ci * blocks_per_chunk * 32;
        LossData L;
        L.Bfull = B; L.A = c->A; L.logstd = distill ? nullptr : c->p + c->logstd; L.idx = rows; L.action = c->action; L.logp_old = c->logp;
        L.v_old = c->value; L.adv = hp->norm_adv ? c->adv_n : c->adv; L.ret = c->ret; L.clip_eps = hp->clip_eps; L.vclip_eps = hp->vclip_eps; L.vf_coef = hp->vf_coef;
        L.aux_dim = distill ? hp->aux_dim : 0; L.aux_coef = hp->aux_coef;
        bool head_done = false;
        if (fused_head) {
          rc = launch_head_loss(c, L, n, c0 > 0, distill, sp, dp);
          if (rc != PPO_OK && rc != 1) return rc;
          head_done = rc == PPO_OK;
          if (!head_done) {  // workspaces too small for the fused form: the output layer as a GEMM after all
            ARows al = plain_arows(c->fcact[c->nfc - 1], c->hid, n, c->hid);
            Ep<MapRows, float, true, false, false> ep;
            ep.map = plain_map(HEAD_LD, n); ep.out = c->headout; ep.bias = c->p + c->headB; ep.mask = nullptr; ep.N = c->NH;
            rc = launch_gemm(c, al, n, c->shadow + c->headW, c->hid, c->NH, c->hid, ep, "head_fwd", 2.0 * n * c->hid + 4.0 * n * c->NH);
            if (rc) return rc;
          }
        }
        if (!head_done) {
        ProfScope ps(c, "loss", 0.0, (double)n * (HEAD_LD * 6.0 + 4.0 * c->A + 20.0));
        if (distill) hipLaunchKernelGGL(k_loss<true>, dim3(cdiv(n, LOSS_BLOCK)), dim3(LOSS_BLOCK), 0, c->stream, n, L, c->headout, c->dhead, sp, dp);
        else hipLaunchKernelGGL(k_loss<false>, dim3(cdiv(n, LOSS_BLOCK)), dim3(LOSS_BLOCK), 0, c->stream, n, L, c->headout, c->dhead, sp, dp);
        LAUNCHCHK(c, "loss kernel");
        }
        // partial slots of a ragged last chunk follow the full chunks contiguously
        nblocks = ci * blocks_per_chunk + cdiv(n, LOSS_BLOCK);
        if (c0 + CU >= Bu) {
          // last chunk: every loss partial of the minibatch exists; their sums (statistics, log-std gradient)
          // are taken by one more block of the backward pass's reduction launch
          LossFinalize& f = c->lossfin;
          f.on = 1; f.nblocks = nblocks; f.Bfull = B; f.A = c->A; f.distill = distill ? 1 : 0; f.stat_part = c->stat_part; f.dls_part = c->dls_part;
          f.logstd = distill ? nullptr : c->p + c->logstd; f.vf_coef = hp->vf_coef; f.ent_coef = hp->ent_coef; f.st = c->dstats + k;
          f.g_logstd = distill ? nullptr : c->g + c->logstd;
          f.desired_kl = adaptive ? hp->desired_kl : 0.f; f.lr_min = hp->lr_min; f.lr_max = hp->lr_max; f.lr_init = hp->lr; f.lr_dev = c->lr_dev;
          f.lr_reset = (k == 0 && !(hp->lr_carry && c->lr_live)) ? 1 : 0;
          f.aux_dim = distill ? hp->aux_dim : 0; f.aux_coef = hp->aux_coef;
        }
        rc = recurrent ? backward_seq_chunk(c, nu, c0 > 0, !head_done) : backward_chunk(c, rows, n, c0 > 0, !head_done);
        if (rc) return rc;
      }
      if (c->lossfin.on) { rc = flush_reduces(c); if (rc) return rc; }  // (a backward pass always ends with a flush; kept for safety)
      c->step += 1;
      {
      ProfScope ps(c, "adam", 0.0, 30.0 * (double)c->total);
      const double c1 = 1.0 - pow((double)hp->beta1, (double)c->step), c2 = 1.0 - pow((double)hp->beta2, (double)c->step);
      const bool clip = hp->max_grad_norm > 0.f;
      if (clip) {  // the norm has to be known before the step: one more pass over the gradient
        hipLaunchKernelGGL(k_gnorm_partial, dim3(c->adam_blocks), dim3(256), 0, c->stream, c->total, c->g, c->sq_part);
        LAUNCHCHK(c, "k_gnorm_partial");
        GnormFinalize gf; gf.on = 1; gf.nb = c->adam_blocks; gf.sq_part = c->sq_part; gf.st = c->dstats + k; gf.max_norm = hp->max_grad_norm; gf.clip_coef = c->clip_coef;
        hipLaunchKernelGGL(k_gnorm_finalize, dim3(1), dim3(256), 0, c->stream, gf);
        LAUNCHCHK(c, "k_gnorm_finalize");
      }
      hipLaunchKernelGGL(k_adam, dim3(c->adam_blocks), dim3(256), 0, c->stream, c->total, c->p, c->m, c->v, c->g, c->shadow, hp->lr, hp->beta1, hp->beta2,
                         hp->adam_eps, (float)(1.0 / c1), (float)(1.0 / c2), c->sq_part, clip ? c->clip_coef : nullptr,
                         adaptive ? c->lr_dev : nullptr);
      LAUNCHCHK(c, "k_adam");
      if (!clip) {  // the step's gradient norm: one more block of the re-pack launch that follows
        GnormFinalize& gf = c->gnfin;
        gf.on = 1; gf.nb = c->adam_blocks; gf.sq_part = c->sq_part; gf.st = c->dstats + k; gf.max_norm = 0.f; gf.clip_coef = nullptr;
      }
      }
      rc = repack_weights(c);
      if (rc) return rc;
    }
  }
  c->update_idx += 1;
  if (adaptive) c->lr_live = true;
  if (host_stats) {
    HIPCHK(c, hipMemcpyAsync(host_stats, c->dstats, sizeof(DevStats) * (size_t)steps, hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  return PPO_OK;
}

int create_impl(Ctx* c) {
  build_geometry(c);
  HIPCHK(c, hipGetDevice(&c->dev));
  if (c->dev < 0 || c->dev >= 64) return fail(c, PPO_EHIP, "device number %d out of range", c->dev);
  { int32_t* ws = nullptr; HIPCHK(c, static_scratch(&ws)); }  // the static scratch of ppo_permutation_static on this device
  const int V = c->V;
  int CH = c->d.max_chunk > 0 ? c->d.max_chunk : 16384 / V;
  if (CH > c->S) CH = c->S;
  if (CH < 1) CH = 1;
  c->CH = CH;
  // the kernels index rows with 32-bit integers
  if ((int64_t)CH * V * c->cH[1] * c->cW[1] >= (1LL << 31) || (int64_t)CH * c->feat_ld >= (1LL << 40))
    return fail(c, PPO_ESHAPE, "chunk of %d samples is too large for 32-bit row indices; lower max_chunk", CH);
  const int64_t S = c->S;
  c->PU = c->nl > 0 ? c->N : c->S;
  c->CHe = CH / c->T < 1 ? 1 : CH / c->T;
  if (c->CHe > c->N) c->CHe = c->N;
  if (c->nl > 0 && (int64_t)c->CHe * c->T > CH) return fail(c, PPO_ESHAPE, "max_chunk = %d holds no whole environment of %d steps", CH, c->T);
  // parameters
  DALLOC(c, c->p, c->total); DALLOC(c, c->m, c->total); DALLOC(c, c->v, c->total); DALLOC(c, c->g, c->total);
  DALLOC(c, c->shadow, c->total + 8);
  for (int l = 1; l < c->nconv; ++l) {
    for (int py = 0; py < 2; ++py) DALLOC(c, c->wd[l][py], (int64_t)2 * c->cC[l] * (1 + py) * 2 * c->cC[l + 1]);
    DALLOC(c, c->wtap[l], (int64_t)9 * c->cC[l] * c->cC[l + 1]);
  }
  for (int l = 0; l < c->nfc; ++l) DALLOC(c, c->fcT[l], (int64_t)c->fin[l] * c->fout[l]);
  DALLOC(c, c->headT, (int64_t)c->hid * HEAD_LD);
  if (c->XH > 0) { DALLOC(c, c->aux1T, (int64_t)c->hid * c->XH); DALLOC(c, c->aux2T, (int64_t)c->XH * HEAD_LD); }
  // rollout buffer
  DALLOC(c, c->obs, S * V * c->img_elems);
  DALLOC(c, c->proprio, S * c->P); DALLOC(c, c->action, S * c->A);
  DALLOC(c, c->logp, S); DALLOC(c, c->value, S); DALLOC(c, c->reward, S); DALLOC(c, c->adv, S); DALLOC(c, c->adv_n, S); DALLOC(c, c->ret, S); DALLOC(c, c->done, S);
  // permutation of the PU units a minibatch is drawn from: about 32 keys per bucket
  int nb = 1, lg = 0;
  while ((int64_t)nb * 32 < c->PU && nb < (1 << 20)) { nb <<= 1; ++lg; }
  c->nb = nb; c->shift = 64 - lg;
  DALLOC(c, c->perm, (int64_t)PERM_BATCH * c->PU); DALLOC(c, c->ptmp, (int64_t)PERM_BATCH * c->PU);  // one slot per epoch of a batch
  DALLOC(c, c->phist, (int64_t)PERM_BATCH * 2 * nb); DALLOC(c, c->pstart, (int64_t)PERM_BATCH * nb);
  // workspaces
  int64_t gmax = (int64_t)CH * c->feat_ld;
  for (int l = 0; l < c->nconv - 1; ++l) {
    int64_t e = (int64_t)CH * V * c->cC[l + 1] * c->cH[l + 1] * c->cW[l + 1];
    DALLOC(c, c->act[l], e);
    DALLOC(c, c->abits[l], (int64_t)CH * V * c->cH[l + 1] * c->cW[l + 1] * ((c->cC[l + 1] + 31) / 32));
    if (e > gmax) gmax = e;
  }
  DALLOC(c, c->feat, (int64_t)CH * c->feat_ld);
  if ((int64_t)CH * c->fin[0] > gmax) gmax = (int64_t)CH * c->fin[0];
  if (c->E > 0) {  // the last convolution's activation has a buffer of its own, read by the embedding
    const int l = c->nconv - 1;
    DALLOC(c, c->act[l], (int64_t)CH * V * c->flat);
    DALLOC(c, c->embT, (int64_t)c->flat * c->E);
    if ((int64_t)CH * V * c->flat > gmax) gmax = (int64_t)CH * V * c->flat;
  }
  if (c->ln) {
    int64_t emax = 0;
    for (int l = 0; l < c->nconv; ++l) {
      const int64_t e = (int64_t)CH * V * c->cC[l + 1] * c->cH[l + 1] * c->cW[l + 1];
      DALLOC(c, c->pre[l], e); DALLOC(c, c->lnstat[l], (int64_t)CH * V);
      if (e > emax) emax = e;
    }
    DALLOC(c, c->dpre, emax);
    if (emax > gmax) gmax = emax;
  }
  if (c->nl > 0) {
    const int H = c->H;
    c->xh[0] = c->feat;
    for (int l = 0; l < c->nl; ++l) {
      const int64_t K = c->lin[l] + H;
      DALLOC(c, c->lstmWT[l], K * 4 * H);
      if (l > 0) DALLOC(c, c->xh[l], (int64_t)CH * K);
      DALLOC(c, c->dxh[l], (int64_t)CH * K);
      DALLOC(c, c->gates[l], (int64_t)CH * 4 * H); DALLOC(c, c->c_enter[l], (int64_t)CH * H);
    }
    DALLOC(c, c->lstm_pre, (int64_t)c->CHe * 4 * H); DALLOC(c, c->da, (int64_t)CH * 4 * H); DALLOC(c, c->dc_carry, (int64_t)c->CHe * H);
    DALLOC(c, c->htop, (int64_t)CH * H); DALLOC(c, c->seqidx, CH);
    DALLOC(c, c->h0, (int64_t)c->nl * c->N * H); DALLOC(c, c->c0, (int64_t)c->nl * c->N * H);
    HIPCHK(c, hipMemsetAsync(c->h0, 0, sizeof(float) * (size_t)c->nl * c->N * H, c->stream));
    HIPCHK(c, hipMemsetAsync(c->c0, 0, sizeof(float) * (size_t)c->nl * c->N * H, c->stream));
    if ((int64_t)CH * H > gmax) gmax = (int64_t)CH * H;
  }
  for (int l = 0; l < c->nfc; ++l) { DALLOC(c, c->fcact[l], (int64_t)CH * c->fout[l]); if ((int64_t)CH * c->fout[l] > gmax) gmax = (int64_t)CH * c->fout[l]; }
  DALLOC(c, c->headout, (int64_t)CH * HEAD_LD); DALLOC(c, c->dhead, (int64_t)CH * HEAD_LD);
  if (c->XH > 0) {
    DALLOC(c, c->auxact, (int64_t)CH * c->XH); DALLOC(c, c->dauxact, (int64_t)CH * c->XH); DALLOC(c, c->daux, (int64_t)CH * HEAD_LD);
    HIPCHK(c, hipMemsetAsync(c->headout, 0, sizeof(float) * (size_t)CH * HEAD_LD, c->stream));
  }
  DALLOC(c, c->gbuf[0], gmax); DALLOC(c, c->gbuf[1], gmax);
  // weight-gradient partials: room for every layer at its preferred split count, all layers of a backward
  // pass side by side (their sums are taken in one launch at the end of the pass)
  int64_t pe_sum = 2048LL * c->cC[1] * (9 * c->cC[0] + 1), bpe_sum = 0;
  auto want = [&](int Nn, int Kk, int64_t M, int64_t& need, int64_t& bneed) {  // k_wgrad
    int ktw = Kk <= 128 ? 1 : (Kk <= 256 ? 2 : 3);
    int tiles = cdiv(Kk, 128 * ktw) * cdiv(Nn, 64);
    int splits = cdiv(768, tiles), mr = cdiv(M, 128);
    if (splits > mr) splits = mr;
    if (splits < 1) splits = 1;
    need = (int64_t)splits * Nn * Kk; bneed = (int64_t)splits * Nn;
  };
  for (int l = 1; l < c->nconv; ++l) {
    int64_t need, bneed;
    want(c->cC[l + 1], 9 * c->cC[l], (int64_t)CH * V * c->cH[l + 1] * c->cW[l + 1], need, bneed);
    // or one partial per block of the LDS-image weight-gradient kernel
    const int64_t gy = cdiv(c->cC[l + 1], 64), gx = 256 / gy > 0 ? 256 / gy : 1, per = (int64_t)c->cC[l + 1] * 9 * c->cC[l];
    if (gx * per > need) need = gx * per;
    if (gx * c->cC[l + 1] > bneed) bneed = gx * c->cC[l + 1];
    pe_sum += need; bpe_sum += bneed;
  }
  for (int l = 0; l < c->nfc; ++l) {
    int64_t need, bneed;
    want(c->fout[l], c->fin[l], CH, need, bneed);
    const int64_t per = (int64_t)c->fout[l] * c->fin[l];  // k_wgrad_rs: up to four splits are worth their partials
    if (4 * per > need) need = 4 * per;
    if (4 * (int64_t)c->fout[l] > bneed) bneed = 4 * (int64_t)c->fout[l];
    pe_sum += need; bpe_sum += bneed;
  }
  {
    int64_t need, bneed;
    want(c->NH, c->hid, CH, need, bneed);
    const int64_t nblk = cdiv(CH, 64);  // fused output-layer kernel: one partial per 64 samples
    if (nblk * c->NH * c->hid > need) need = nblk * c->NH * c->hid;
    if (nblk * c->NH > bneed) bneed = nblk * c->NH;
    pe_sum += need; bpe_sum += bneed;
  }
  if (c->E > 0) { int64_t need, bneed; want(c->E, c->flat, CH, need, bneed); pe_sum += need; bpe_sum += bneed; }
  for (int l = 0; l < c->nl; ++l) {
    int64_t need, bneed;
    want(4 * c->H, c->lin[l] + c->H, CH, need, bneed);
    const int64_t per = (int64_t)4 * c->H * (c->lin[l] + c->H);
    if (4 * per > need) need = 4 * per;
    if (16 * (int64_t)c->H > bneed) bneed = 16 * (int64_t)c->H;
    pe_sum += need; bpe_sum += bneed;
  }
  if (c->ln) pe_sum += 1024LL * 2 * 1024;  // layer-norm gain / shift partials: one per block of k_ln_bwd
  if (c->XH > 0) {
    int64_t need, bneed;
    want(c->XH, c->hid, CH, need, bneed); pe_sum += need; bpe_sum += bneed;
    want(c->X, c->XH, CH, need, bneed); pe_sum += need; bpe_sum += bneed;
  }
  c->partial_cap = pe_sum; c->bias_partial_cap = bpe_sum > 0 ? bpe_sum : 1;
  DALLOC(c, c->partial_base, c->partial_cap); DALLOC(c, c->bias_partial_base, c->bias_partial_cap);
  c->partial = c->partial_base; c->partial_elems = c->partial_cap;
  c->bias_partial = c->bias_partial_base; c->bias_partial_elems = c->bias_partial_cap;
  c->rjobs.njobs = 0; c->rjob_blocks = 0;
  DALLOC(c, c->zpage, 32768);
  HIPCHK(c, hipMemsetAsync(c->zpage, 0, 65536, c->stream));
  // loss / Adam partials
  {
    const int CU = c->nl > 0 ? c->CHe : CH, Lr = c->nl > 0 ? c->T : 1;
    c->max_loss_blocks = (cdiv(c->PU, CU) + 1) * cdiv((int64_t)CU * Lr, LOSS_BLOCK) + 1;
  }
  DALLOC(c, c->stat_part, (int64_t)c->max_loss_blocks * LOSS_NSTAT); DALLOC(c, c->dls_part, (int64_t)c->max_loss_blocks * 32);
  c->adam_blocks = cdiv(c->total, 1024); if (c->adam_blocks > 2048) c->adam_blocks = 2048;
  DALLOC(c, c->sq_part, c->adam_blocks);
  DALLOC(c, c->clip_coef, 1); DALLOC(c, c->lr_dev, 1); DALLOC(c, c->advn_part, 3 * ADVN_BLOCKS);
  DALLOC(c, c->dstats, c->max_steps);
  HIPCHK(c, hipMemsetAsync(c->p, 0, sizeof(float) * (size_t)c->total, c->stream));
  HIPCHK(c, hipMemsetAsync(c->m, 0, sizeof(float) * (size_t)c->total, c->stream));
  HIPCHK(c, hipMemsetAsync(c->v, 0, sizeof(float) * (size_t)c->total, c->stream));
  HIPCHK(c, hipMemsetAsync(c->g, 0, sizeof(float) * (size_t)c->total, c->stream));
  HIPCHK(c, hipMemsetAsync(c->shadow, 0, sizeof(bf16_t) * (size_t)(c->total + 8), c->stream));
  int rc = refresh_shadow(c);
  if (rc) return rc;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->written.assign((size_t)c->T, 0);
  c->cover.assign((size_t)c->T, {});
  return PPO_OK;
}

void free_all(Ctx* c) {
  for (void* p : c->allocs) (void)hipFree(p);
  c->allocs.clear();
}

int to_internal(Ctx* c, const float* canon, float* dev) {
  std::vector<float> tmp((size_t)c->total);
  for (int64_t i = 0; i < c->total; ++i) tmp[(size_t)i] = canon[c->i2c[(size_t)i]];
  HIPCHK(c, hipMemcpyAsync(dev, tmp.data(), sizeof(float) * (size_t)c->total, hipMemcpyHostToDevice, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return PPO_OK;
}
int to_canonical(Ctx* c, const float* dev, float* canon) {
  std::vector<float> tmp((size_t)c->total);
  HIPCHK(c, hipMemcpyAsync(tmp.data(), dev, sizeof(float) * (size_t)c->total, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (int64_t i = 0; i < c->total; ++i) canon[c->i2c[(size_t)i]] = tmp[(size_t)i];
  return PPO_OK;
}

}  // namespace

struct ppo_ctx : Ctx {};

extern "C" {

int ppo_create(ppo_ctx** out, const ppo_net_desc* desc, void* hip_stream) {
  if (!out) return fail(nullptr, PPO_EINVAL, "out is NULL");
  *out = nullptr;
  int rc = validate_desc(desc);
  if (rc) return rc;
  ppo_ctx* c = new (std::nothrow) ppo_ctx();
  if (!c) return fail(nullptr, PPO_ENOMEM, "host allocation failed");
  c->d = *desc;
  c->stream = (hipStream_t)hip_stream;
  rc = create_impl(c);
  if (rc) { g_create_error = c->err; free_all(c); delete c; return rc; }
  *out = c;
  return PPO_OK;
}

int ppo_destroy(ppo_ctx* c) {
  if (!c) return PPO_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  for (auto& r : c->prof_recs) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
  for (auto e : c->prof_pool) (void)hipEventDestroy(e);
  free_all(c);
  delete c;
  return PPO_OK;
}

const char* ppo_last_error(const ppo_ctx* c) { return c ? c->err.c_str() : g_create_error.c_str(); }

int64_t ppo_param_count(const ppo_ctx* c) { return c ? c->total : PPO_EINVAL; }
int64_t ppo_buffer_image_bytes(const ppo_ctx* c) { return c ? (int64_t)c->S * c->V * c->img_elems * (int64_t)sizeof(bf16_t) : PPO_EINVAL; }

int ppo_set_params(ppo_ctx* c, const float* h, int64_t n) {
  if (!c) return PPO_EINVAL;
  if (!h) return fail(c, PPO_EINVAL, "h_params is NULL");
  if (n != c->total) return fail(c, PPO_ESHAPE, "expected %lld parameters, got %lld", (long long)c->total, (long long)n);
  int rc = to_internal(c, h, c->p);
  if (rc) return rc;
  rc = refresh_shadow(c);
  if (rc) return rc;
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return PPO_OK;
}
int ppo_get_params(ppo_ctx* c, float* h, int64_t n) {
  if (!c) return PPO_EINVAL;
  if (!h) return fail(c, PPO_EINVAL, "h_params is NULL");
  if (n != c->total) return fail(c, PPO_ESHAPE, "expected %lld parameters, got %lld", (long long)c->total, (long long)n);
  return to_canonical(c, c->p, h);
}
int ppo_get_grads(ppo_ctx* c, float* h, int64_t n) {
  if (!c) return PPO_EINVAL;
  if (!h) return fail(c, PPO_EINVAL, "h_grads is NULL");
  if (n != c->total) return fail(c, PPO_ESHAPE, "expected %lld parameters, got %lld", (long long)c->total, (long long)n);
  return to_canonical(c, c->g, h);
}
int ppo_set_opt_state(ppo_ctx* c, const float* hm, const float* hv, int64_t n, int64_t step, int64_t update_idx) {
  if (!c) return PPO_EINVAL;
  if (!hm || !hv) return fail(c, PPO_EINVAL, "h_m / h_v is NULL");
  if (n != c->total) return fail(c, PPO_ESHAPE, "expected %lld parameters, got %lld", (long long)c->total, (long long)n);
  if (step < 0 || update_idx < 0) return fail(c, PPO_EINVAL, "step and update_idx must be >= 0");
  int rc = to_internal(c, hm, c->m);
  if (rc) return rc;
  rc = to_internal(c, hv, c->v);
  if (rc) return rc;
  c->step = step; c->update_idx = update_idx;
  return PPO_OK;
}
int ppo_get_opt_state(ppo_ctx* c, float* hm, float* hv, int64_t n, int64_t* step, int64_t* update_idx) {
  if (!c) return PPO_EINVAL;
  if (!hm || !hv) return fail(c, PPO_EINVAL, "h_m / h_v is NULL");
  if (n != c->total) return fail(c, PPO_ESHAPE, "expected %lld parameters, got %lld", (long long)c->total, (long long)n);
  int rc = to_canonical(c, c->m, hm);
  if (rc) return rc;
  rc = to_canonical(c, c->v, hv);
  if (rc) return rc;
  if (step) *step = c->step;
  if (update_idx) *update_idx = c->update_idx;
  return PPO_OK;
}

int ppo_get_adaptive_lr(ppo_ctx* c, float* h_lr, int32_t* h_live) {
  if (!c) return PPO_EINVAL;
  if (!h_lr || !h_live) return fail(c, PPO_EINVAL, "h_lr / h_live is NULL");
  *h_live = c->lr_live ? 1 : 0;
  *h_lr = 0.f;
  if (c->lr_live) {
    HIPCHK(c, hipMemcpyAsync(h_lr, c->lr_dev, sizeof(float), hipMemcpyDeviceToHost, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  return PPO_OK;
}
int ppo_set_adaptive_lr(ppo_ctx* c, float lr, int32_t live) {
  if (!c) return PPO_EINVAL;
  if (live != 0 && live != 1) return fail(c, PPO_EINVAL, "live must be 0 or 1");
  if (live && !(isfinite(lr) && lr > 0.f)) return fail(c, PPO_EINVAL, "a live adaptive rate must be finite and > 0");
  if (live) {
    HIPCHK(c, hipMemcpyAsync(c->lr_dev, &lr, sizeof(float), hipMemcpyHostToDevice, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  c->lr_live = live != 0;
  return PPO_OK;
}

static int write_slab(ppo_ctx* c, int32_t t, int32_t n0, int32_t cnt, const void* d_obs, const float* d_proprio, const float* d_action,
                      const float* d_logp, const float* d_value, const float* d_reward, const uint8_t* d_done);
static int all_written(ppo_ctx* c);

int ppo_buffer_write(ppo_ctx* c, int32_t t, const void* d_obs, const float* d_proprio, const float* d_action, const float* d_logp,
                     const float* d_value, const float* d_reward, const uint8_t* d_done) {
  if (!c) return PPO_EINVAL;
  if (t < 0 || t >= c->T) return fail(c, PPO_EINVAL, "t = %d outside [0, %d)", t, c->T);
  if (!d_obs || !d_proprio || !d_action) return fail(c, PPO_EINVAL, "d_obs, d_proprio and d_action must not be NULL");
  if (c->d.has_value_head && (!d_logp || !d_value || !d_reward || !d_done))
    return fail(c, PPO_EINVAL, "an actor-critic buffer needs d_logp, d_value, d_reward and d_done");
  const int rc = write_slab(c, t, 0, c->N, d_obs, d_proprio, d_action, d_logp, d_value, d_reward, d_done);
  if (rc) return rc;
  if (t == 0) { c->written.assign((size_t)c->T, 0); c->cover.assign((size_t)c->T, {}); }
  c->written[(size_t)t] = 1;
  c->cover[(size_t)t].clear();
  c->gae_done = false;
  return PPO_OK;
}

int ppo_buffer_write_range(ppo_ctx* c, int32_t t, int32_t env_offset, int32_t count, const void* d_obs, const float* d_proprio,
                           const float* d_action, const float* d_logp, const float* d_value, const float* d_reward, const uint8_t* d_done) {
  if (!c) return PPO_EINVAL;
  if (t < 0 || t >= c->T) return fail(c, PPO_EINVAL, "t = %d outside [0, %d)", t, c->T);
  if (env_offset < 0 || count < 0 || (int64_t)env_offset + count > c->N)
    return fail(c, PPO_EINVAL, "environments [%d, %d + %d) outside [0, %d)", env_offset, env_offset, count, c->N);
  if (count == 0) return PPO_OK;
  if (!d_obs || !d_proprio || !d_action) return fail(c, PPO_EINVAL, "d_obs, d_proprio and d_action must not be NULL");
  if (c->d.has_value_head && (!d_logp || !d_value || !d_reward || !d_done))
    return fail(c, PPO_EINVAL, "an actor-critic buffer needs d_logp, d_value, d_reward and d_done");
  // a range that arrives while every step of the rollout is complete is the first slice of the NEXT rollout: from
  // here on no step counts as written until its own ranges have covered [0, N) again (the slabs still hold the
  // previous rollout's records)
  const bool new_rollout = all_written(c) != 0;
  const int rc = write_slab(c, t, env_offset, count, d_obs, d_proprio, d_action, d_logp, d_value, d_reward, d_done);
  if (rc) return rc;
  if (new_rollout) { c->written.assign((size_t)c->T, 0); c->cover.assign((size_t)c->T, {}); }
  // within a rollout, a write into a complete step starts that step afresh; the step is complete again once the
  // ranges cover [0, N)
  auto& cv = c->cover[(size_t)t];
  if (c->written[(size_t)t] == 1) cv.clear();
  cv.push_back({env_offset, env_offset + count});
  std::sort(cv.begin(), cv.end());
  std::vector<std::pair<int, int>> merged;
  for (const auto& r : cv) {
    if (!merged.empty() && r.first <= merged.back().second) merged.back().second = std::max(merged.back().second, r.second);
    else merged.push_back(r);
  }
  cv.swap(merged);
  const bool complete = cv.size() == 1 && cv[0].first == 0 && cv[0].second == c->N;
  c->written[(size_t)t] = complete ? 1 : 0;
  if (complete) cv.clear();
  c->gae_done = false;
  return PPO_OK;
}

int ppo_buffer_write_state(ppo_ctx* c, const float* d_h0, const float* d_c0) {
  if (!c) return PPO_EINVAL;
  if (c->nl <= 0) return fail(c, PPO_ESTATE, "this network has no recurrent layers");
  const size_t bytes = sizeof(float) * (size_t)c->nl * c->N * c->H;
  if (d_h0) HIPCHK(c, hipMemcpyAsync(c->h0, d_h0, bytes, hipMemcpyDeviceToDevice, c->stream));
  else HIPCHK(c, hipMemsetAsync(c->h0, 0, bytes, c->stream));
  if (d_c0) HIPCHK(c, hipMemcpyAsync(c->c0, d_c0, bytes, hipMemcpyDeviceToDevice, c->stream));
  else HIPCHK(c, hipMemsetAsync(c->c0, 0, bytes, c->stream));
  return PPO_OK;
}

int ppo_buffer_read_obs(ppo_ctx* c, int32_t t, void* d_obs_bf16) {
  if (!c) return PPO_EINVAL;
  if (t < 0 || t >= c->T) return fail(c, PPO_EINVAL, "t = %d outside [0, %d)", t, c->T);
  if (!d_obs_bf16) return fail(c, PPO_EINVAL, "d_obs_bf16 is NULL");
  if (!c->written[(size_t)t]) return fail(c, PPO_ESTATE, "step %d has not been written", t);
  const int64_t nimg = (int64_t)c->N * c->V, n = nimg * c->img_elems;
  hipLaunchKernelGGL(k_read_obs, dim3(cdiv(n, 256)), dim3(256), 0, c->stream, c->obs + (int64_t)t * n, (bf16_t*)d_obs_bf16, nimg, c->d.in_c,
                     c->d.in_h * c->d.in_w);
  LAUNCHCHK(c, "k_read_obs");
  return PPO_OK;
}

static int all_written(ppo_ctx* c) {
  for (char w : c->written) if (w != 1) return 0;  // 2: acted, outcome still missing
  return 1;
}

// Images, proprioception and (where given) the other fields of step t into the slab: one launch.
// Environments [n0, n0 + cnt) of the step; the caller's arrays hold cnt rows.
static int write_slab(ppo_ctx* c, int32_t t, int32_t n0, int32_t cnt, const void* d_obs, const float* d_proprio, const float* d_action,
                      const float* d_logp, const float* d_value, const float* d_reward, const uint8_t* d_done) {
  const int N = cnt, V = c->V, HW = c->d.in_h * c->d.in_w, C = c->d.in_c;
  const int64_t nimg = (int64_t)N * V, groups = (HW + 7) / 8;
  const int64_t off = (int64_t)t * c->N + n0;
  bf16_t* dst = c->obs + off * V * c->img_elems;
  ProfScope ps(c, "buffer_write", 0.0, (double)nimg * c->img_elems * (c->d.obs_dtype == 0 ? 6.0 : 4.0) + (double)N * (6.0 * c->P + 8.0 * c->A + 26.0));
  const int mx = c->P > c->A ? c->P : c->A;
  ScalarWrite sw;
  sw.N = N; sw.P = c->P; sw.A = c->A; sw.proprio = d_proprio; sw.action = d_action; sw.logp = d_logp; sw.value = d_value; sw.reward = d_reward; sw.done = d_done;
  sw.o_proprio = c->proprio + off * c->P; sw.o_action = c->action + off * c->A; sw.o_logp = c->logp + off; sw.o_value = c->value + off;
  sw.o_reward = c->reward + off; sw.o_done = c->done + off;
  const int obs_blocks = cdiv(nimg * groups, 256), sc_blocks = cdiv((int64_t)N * mx, 256);
  if (c->d.obs_dtype == 0)
    hipLaunchKernelGGL((k_write_obs<float>), dim3(obs_blocks + sc_blocks), dim3(256), 0, c->stream, (const float*)d_obs, dst, nimg, C, HW, obs_blocks, sw);
  else
    hipLaunchKernelGGL((k_write_obs<bf16_t>), dim3(obs_blocks + sc_blocks), dim3(256), 0, c->stream, (const bf16_t*)d_obs, dst, nimg, C, HW, obs_blocks, sw);
  LAUNCHCHK(c, "k_write_obs");
  return PPO_OK;
}

int ppo_gae(ppo_ctx* c, const float* d_last_value, float gamma, float lambda) {
  if (!c) return PPO_EINVAL;
  if (!d_last_value) return fail(c, PPO_EINVAL, "d_last_value is NULL");
  if (!isfinite(gamma) || !isfinite(lambda) || gamma < 0.f || gamma > 1.f || lambda < 0.f || lambda > 1.f)
    return fail(c, PPO_EINVAL, "gamma and lambda must be in [0, 1]");
  if (!c->d.has_value_head) return fail(c, PPO_ESTATE, "this context has no value head (distillation student)");
  if (!all_written(c)) return fail(c, PPO_ESTATE, "ppo_gae needs all %d steps written", c->T);
  ProfScope ps(c, "gae", 6.0 * c->S, 17.0 * c->S + 4.0 * c->N);
  if (c->T <= 8) hipLaunchKernelGGL(k_gae<8>, dim3(cdiv(c->N, 64)), dim3(64), 0, c->stream, c->T, c->N, c->reward, c->done, c->value, d_last_value, gamma, lambda, c->adv, c->ret);
  else if (c->T <= 16) hipLaunchKernelGGL(k_gae<16>, dim3(cdiv(c->N, 64)), dim3(64), 0, c->stream, c->T, c->N, c->reward, c->done, c->value, d_last_value, gamma, lambda, c->adv, c->ret);
  else hipLaunchKernelGGL(k_gae<32>, dim3(cdiv(c->N, 64)), dim3(64), 0, c->stream, c->T, c->N, c->reward, c->done, c->value, d_last_value, gamma, lambda, c->adv, c->ret);
  LAUNCHCHK(c, "k_gae");
  c->gae_done = true;
  return PPO_OK;
}

int ppo_get_adv_ret(ppo_ctx* c, float* d_adv, float* d_ret) {
  if (!c) return PPO_EINVAL;
  if (!c->gae_done) return fail(c, PPO_ESTATE, "ppo_gae has not run on this rollout");
  if (d_adv) HIPCHK(c, hipMemcpyAsync(d_adv, c->adv, sizeof(float) * (size_t)c->S, hipMemcpyDeviceToDevice, c->stream));
  if (d_ret) HIPCHK(c, hipMemcpyAsync(d_ret, c->ret, sizeof(float) * (size_t)c->S, hipMemcpyDeviceToDevice, c->stream));
  return PPO_OK;
}

int ppo_permutation(ppo_ctx* c, uint64_t seed, uint64_t update_idx, uint64_t epoch, int32_t* h_perm) {
  if (!c) return PPO_EINVAL;
  if (!h_perm) return fail(c, PPO_EINVAL, "h_perm is NULL");
  int rc = gen_permutation(c, seed, update_idx, epoch);
  if (rc) return rc;
  HIPCHK(c, hipMemcpyAsync(h_perm, c->perm, sizeof(int32_t) * (size_t)c->PU, hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  return PPO_OK;
}

int ppo_permutation_static(int64_t S, uint64_t seed, uint64_t update_idx, uint64_t epoch, int32_t* d_perm, void* hip_stream) {
  if (S < 0) return fail(nullptr, PPO_EINVAL, "S must be >= 0");
  if (S > STATIC_PERM_MAX_S)
    return fail(nullptr, PPO_ESHAPE, "ppo_permutation_static handles at most %lld samples (got %lld); use a context's ppo_permutation",
                (long long)STATIC_PERM_MAX_S, (long long)S);
  if (S == 0) return PPO_OK;
  if (!d_perm) return fail(nullptr, PPO_EINVAL, "d_perm is NULL");
  int32_t* ws = nullptr;
  {
    const hipError_t e = static_scratch(&ws);
    if (e != hipSuccess) return fail(nullptr, PPO_EHIP, "address of the static scratch array: %s", hipGetErrorString(e));
  }
  // the bucket count of ppo_create (about 32 keys per bucket), so both entry points run the same kernels on the same grids
  int nb = 1, lg = 0;
  while ((int64_t)nb * 32 < S && nb < STATIC_PERM_MAX_NB) { nb <<= 1; ++lg; }
  const int shift = 64 - lg;
  int32_t* hist = ws;                  // [2 * nb]: counts, then scatter cursors
  int32_t* start = ws + 2 * (int64_t)STATIC_PERM_MAX_NB;  // [nb]
  int32_t* tmp = ws + 3 * (int64_t)STATIC_PERM_MAX_NB;    // [S]
  hipStream_t st = (hipStream_t)hip_stream;
  PermStreams ps;
  for (int e = 0; e < PERM_BATCH; ++e) ps.s[e] = perm_stream(seed, update_idx, epoch);
  const int g = cdiv(S, 256), Si = (int)S;
  // the array keeps the last call's contents: counts and cursors must start at zero (a fill kernel, so that a
  // caller may record this call into a graph); start and tmp are fully overwritten before they are read
  hipLaunchKernelGGL(k_fill_i32, dim3(cdiv((int64_t)2 * nb, 256)), dim3(256), 0, st, hist, (int64_t)2 * nb, 0);
  hipLaunchKernelGGL(k_perm_hist, dim3(g, 1), dim3(256), 0, st, ps, Si, shift, nb, hist);
  hipLaunchKernelGGL(k_perm_scan, dim3(1, 1), dim3(1024), 0, st, hist, start, nb);
  hipLaunchKernelGGL(k_perm_scatter, dim3(g, 1), dim3(256), 0, st, ps, Si, shift, nb, start, hist, tmp);
  hipLaunchKernelGGL(k_perm_rank, dim3(g, 1), dim3(256), 0, st, ps, Si, shift, nb, start, hist, tmp, d_perm);
  LAUNCHCHK(nullptr, "permutation kernels");
  return PPO_OK;
}

int ppo_update(ppo_ctx* c, const ppo_hparams* hp, ppo_mb_stats* host_stats) {
  if (!c) return PPO_EINVAL;
  if (!c->d.has_value_head) return fail(c, PPO_ESTATE, "ppo_update needs a value head; use distill_update for a student");
  int rc = validate_hp(c, hp, false);
  if (rc) return rc;
  if (!c->gae_done) return fail(c, PPO_ESTATE, "ppo_update needs ppo_gae on the current rollout");
  return run_update(c, hp, host_stats, false);
}

int distill_update(ppo_ctx* c, const ppo_hparams* hp, ppo_mb_stats* host_stats) {
  if (!c) return PPO_EINVAL;
  if (c->d.has_value_head) return fail(c, PPO_ESTATE, "distill_update needs a student context (has_value_head = 0)");
  int rc = validate_hp(c, hp, true);
  if (rc) return rc;
  if (!all_written(c)) return fail(c, PPO_ESTATE, "distill_update needs all %d steps written", c->T);
  return run_update(c, hp, host_stats, true);
}

__global__ void k_copy_heads(int n, int A, int has_v, const float* __restrict__ out, float* __restrict__ mu, float* __restrict__ v) {
  int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= (int64_t)n * HEAD_LD) return;
  int b = (int)(i / HEAD_LD), j = (int)(i - (int64_t)b * HEAD_LD);
  if (j < A) mu[(int64_t)b * A + j] = out[i];
  else if (j == A && has_v && v) v[b] = out[i];
}

int ppo_forward(ppo_ctx* c, const int32_t* d_idx, int64_t count, float* d_mu, float* d_v) {
  if (!c) return PPO_EINVAL;
  if (!d_mu) return fail(c, PPO_EINVAL, "d_mu is NULL");
  if (count < 0 || (!d_idx && count > c->S)) return fail(c, PPO_EINVAL, "count out of range");
  if (c->nl > 0) return fail(c, PPO_ESTATE, "ppo_forward treats samples independently: not available for a recurrent net");
  if (!all_written(c)) return fail(c, PPO_ESTATE, "ppo_forward needs all %d steps written", c->T);
  for (int64_t c0 = 0; c0 < count; c0 += c->CH) {
    int n = (int)((count - c0 < c->CH) ? count - c0 : c->CH);
    const int32_t* idx = d_idx ? d_idx + c0 : nullptr;
    int rc = forward_chunk(c, idx, n, true, c0);  // without indices: samples c0 .. c0 + n - 1
    if (rc) return rc;
    hipLaunchKernelGGL(k_copy_heads, dim3(cdiv((int64_t)n * HEAD_LD, 256)), dim3(256), 0, c->stream, n, c->A, c->d.has_value_head, c->headout,
                       d_mu + c0 * c->A, d_v ? d_v + c0 : nullptr);
    LAUNCHCHK(c, "k_copy_heads");
  }
  return PPO_OK;
}

int ppo_act(ppo_ctx* c, int32_t t, const void* d_obs, const float* d_proprio, const float* d_noise, float* d_action, float* d_logp,
            float* d_value) {
  if (!c) return PPO_EINVAL;
  if (!c->d.has_value_head) return fail(c, PPO_ESTATE, "ppo_act needs an actor-critic context (has_value_head = 1)");
  if (c->nl > 0) return fail(c, PPO_ESTATE, "ppo_act keeps no recurrent state between calls: not available for a recurrent net");
  if (t < 0 || t >= c->T) return fail(c, PPO_EINVAL, "t = %d outside [0, %d)", t, c->T);
  if (!d_obs || !d_proprio || !d_noise) return fail(c, PPO_EINVAL, "d_obs, d_proprio and d_noise must not be NULL");
  int rc = write_slab(c, t, 0, c->N, d_obs, d_proprio, nullptr, nullptr, nullptr, nullptr, nullptr);
  if (rc) return rc;
  if (t == 0) { c->written.assign((size_t)c->T, 0); c->cover.assign((size_t)c->T, {}); }
  c->written[(size_t)t] = 2;
  c->cover[(size_t)t].clear();
  c->gae_done = false;
  const int64_t first = (int64_t)t * c->N;
  for (int64_t c0 = 0; c0 < c->N; c0 += c->CH) {
    const int n = (int)((c->N - c0 < c->CH) ? c->N - c0 : c->CH);
    rc = forward_chunk(c, nullptr, n, true, first + c0);
    if (rc) return rc;
    ProfScope ps(c, "act_sample", 0.0, (double)n * (4.0 * HEAD_LD + 12.0 * c->A + 8.0));
    const int64_t s0 = first + c0;
    hipLaunchKernelGGL(k_act_sample, dim3(cdiv(n, 64)), dim3(64), 0, c->stream, n, c->A, c->headout, c->p + c->logstd, d_noise + c0 * c->A,
                       c->action + s0 * c->A, c->logp + s0, c->value + s0, d_action ? d_action + c0 * c->A : nullptr,
                       d_logp ? d_logp + c0 : nullptr, d_value ? d_value + c0 : nullptr);
    LAUNCHCHK(c, "k_act_sample");
  }
  return PPO_OK;
}

int ppo_buffer_write_outcome(ppo_ctx* c, int32_t t, const float* d_reward, const uint8_t* d_done) {
  if (!c) return PPO_EINVAL;
  if (t < 0 || t >= c->T) return fail(c, PPO_EINVAL, "t = %d outside [0, %d)", t, c->T);
  if (!d_reward || !d_done) return fail(c, PPO_EINVAL, "d_reward and d_done must not be NULL");
  if (!c->written[(size_t)t]) return fail(c, PPO_ESTATE, "step %d holds no record yet (ppo_act or ppo_buffer_write first)", t);
  hipLaunchKernelGGL(k_write_outcome, dim3(cdiv(c->N, 256)), dim3(256), 0, c->stream, c->N, d_reward, d_done, c->reward + (int64_t)t * c->N,
                     c->done + (int64_t)t * c->N);
  LAUNCHCHK(c, "k_write_outcome");
  c->written[(size_t)t] = 1;
  c->gae_done = false;
  return PPO_OK;
}

int ppo_profile(ppo_ctx* c, int32_t enable) {
  if (!c) return PPO_EINVAL;
  (void)hipStreamSynchronize(c->stream);
  for (auto& r : c->prof_recs) { c->prof_pool.push_back(r.a); c->prof_pool.push_back(r.b); }
  c->prof_recs.clear(); c->prof_cls.clear(); c->prof_idx.clear();
  c->prof_on = enable != 0;
  return PPO_OK;
}

int64_t ppo_profile_report(ppo_ctx* c, char* buf, int64_t cap) {
  if (!c || !buf || cap < 1) return PPO_EINVAL;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c, PPO_EHIP, "hipStreamSynchronize failed");
  std::vector<double> ms(c->prof_cls.size(), 0.0);
  for (auto& r : c->prof_recs) {
    float t = 0.f;
    if (hipEventElapsedTime(&t, r.a, r.b) == hipSuccess) ms[(size_t)r.cls] += t;
  }
  std::string out;
  char line[256];
  for (size_t i = 0; i < c->prof_cls.size(); ++i) {
    const auto& pc = c->prof_cls[i];
    snprintf(line, sizeof line, "%s %lld %.6f %.6e %.6e\n", pc.name.c_str(), (long long)pc.launches, ms[i], pc.flops, pc.bytes);
    out += line;
  }
  if ((int64_t)out.size() + 1 > cap) return fail(c, PPO_EINVAL, "report needs %zu bytes", out.size() + 1);
  memcpy(buf, out.c_str(), out.size() + 1);
  return (int64_t)out.size();
}

int ppo_diag_gemm(int32_t M, int32_t N, int32_t K, const float* h_a, const float* h_b, float* h_c) {
  if (!h_a || !h_b || !h_c || M < 1 || N < 1 || K < 8 || K % 8) return PPO_EINVAL;
  Ctx tmp;
  Ctx* c = &tmp;
  if (hipGetDevice(&c->dev) != hipSuccess || c->dev < 0 || c->dev >= 64) return fail(nullptr, PPO_EHIP, "no usable HIP device");
  float *da = nullptr, *db = nullptr, *dc = nullptr;
  bf16_t *ba = nullptr, *bb = nullptr;
  int rc = PPO_OK;
  auto body = [&]() -> int {
    DALLOC(c, da, (int64_t)M * K); DALLOC(c, db, (int64_t)N * K); DALLOC(c, dc, (int64_t)M * N);
    DALLOC(c, ba, (int64_t)M * K); DALLOC(c, bb, (int64_t)N * K);
    DALLOC(c, c->zpage, 32768);
    HIPCHK(c, hipMemset(c->zpage, 0, 65536));
    HIPCHK(c, hipMemcpy(da, h_a, sizeof(float) * (size_t)M * K, hipMemcpyHostToDevice));
    HIPCHK(c, hipMemcpy(db, h_b, sizeof(float) * (size_t)N * K, hipMemcpyHostToDevice));
    hipLaunchKernelGGL(k_cast_bf16, dim3(cdiv((int64_t)M * K, 256)), dim3(256), 0, c->stream, da, ba, (int64_t)M * K);
    hipLaunchKernelGGL(k_cast_bf16, dim3(cdiv((int64_t)N * K, 256)), dim3(256), 0, c->stream, db, bb, (int64_t)N * K);
    LAUNCHCHK(c, "k_cast_bf16");
    ARows al = plain_arows(ba, K, M, K);
    Ep<MapRows, float, false, false, false> ep;
    ep.map = plain_map(N, M); ep.out = dc; ep.bias = nullptr; ep.mask = nullptr; ep.N = N;
    int r = launch_gemm(c, al, M, bb, K, N, K, ep, "diag_gemm", 0.0);
    if (r) return r;
    HIPCHK(c, hipDeviceSynchronize());
    HIPCHK(c, hipMemcpy(h_c, dc, sizeof(float) * (size_t)M * N, hipMemcpyDeviceToHost));
    return PPO_OK;
  };
  rc = body();
  if (rc) g_create_error = c->err;
  free_all(c);
  return rc;
}

int ppo_diag_peak(int32_t kind, int64_t nbytes, int32_t iters, float* h_result) {
  if (!h_result || kind < PEAK_COPY || kind > PEAK_MFMA_VALU || iters < 1 || iters > 100000) return fail(nullptr, PPO_EINVAL, "ppo_diag_peak: bad argument");
  const bool streams = kind != PEAK_MFMA && kind != PEAK_MFMA_VALU;
  if (streams && (nbytes < (1 << 20) || nbytes > (16LL << 30) || nbytes % 16)) return fail(nullptr, PPO_EINVAL, "ppo_diag_peak: nbytes must be a multiple of 16 in [1 MiB, 16 GiB]");
  if (kind == PEAK_MFMA_VALU && (nbytes < 0 || nbytes > 8)) return fail(nullptr, PPO_EINVAL, "ppo_diag_peak: kind 5 takes the number of vector instructions per MFMA (0..8) in nbytes");
  Ctx tmp;
  Ctx* c = &tmp;
  auto body = [&]() -> int {
    uint4 *src = nullptr, *dst = nullptr;
    float* sink = nullptr;
    hipEvent_t e0, e1;
    DALLOC(c, sink, 4);
    const int64_t n16 = nbytes / 16;
    if (streams) {
      DALLOC(c, src, n16); DALLOC(c, dst, n16);
      HIPCHK(c, hipMemset(src, 0, (size_t)nbytes));
      HIPCHK(c, hipMemset(dst, 0, (size_t)nbytes));
    }
    HIPCHK(c, hipEventCreate(&e0)); HIPCHK(c, hipEventCreate(&e1));
    const int mfma_rounds = 4096;
    auto launch = [&]() {
      const dim3 grid(256 * 16), blk(256);
      switch (kind) {
        case PEAK_COPY: hipLaunchKernelGGL(k_peak_stream<PEAK_COPY>, grid, blk, 0, nullptr, src, dst, n16, (uint32_t*)sink); break;
        case PEAK_READ: hipLaunchKernelGGL(k_peak_stream<PEAK_READ>, grid, blk, 0, nullptr, src, dst, n16, (uint32_t*)sink); break;
        case PEAK_WRITE: hipLaunchKernelGGL(k_peak_stream<PEAK_WRITE>, grid, blk, 0, nullptr, src, dst, n16, (uint32_t*)sink); break;
        case PEAK_COPY_NT: hipLaunchKernelGGL(k_peak_stream<PEAK_COPY_NT>, grid, blk, 0, nullptr, src, dst, n16, (uint32_t*)sink); break;
        case PEAK_MFMA: hipLaunchKernelGGL(k_peak_mfma, dim3(256 * 2), dim3(512), 0, nullptr, mfma_rounds, sink); break;
        default:
          switch ((int)nbytes) {
#define PEAK_MV(K_) case K_: hipLaunchKernelGGL(k_peak_mfma_valu<K_>, dim3(256), dim3(512), 0, nullptr, mfma_rounds, sink); break;
            PEAK_MV(0) PEAK_MV(1) PEAK_MV(2) PEAK_MV(3) PEAK_MV(4) PEAK_MV(5) PEAK_MV(6) PEAK_MV(7) PEAK_MV(8)
#undef PEAK_MV
          }
          break;
      }
    };
    for (int i = 0; i < 2; ++i) launch();
    LAUNCHCHK(c, "peak kernel");
    HIPCHK(c, hipEventRecord(e0, nullptr));
    for (int i = 0; i < iters; ++i) launch();
    HIPCHK(c, hipEventRecord(e1, nullptr));
    HIPCHK(c, hipEventSynchronize(e1));
    LAUNCHCHK(c, "peak kernel");
    float ms = 0.f;
    HIPCHK(c, hipEventElapsedTime(&ms, e0, e1));
    (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
    const double sec = (double)ms * 1e-3 / iters;
    if (kind == PEAK_MFMA) *h_result = (float)(256.0 * 2 * 8 * mfma_rounds * 4 * 32768.0 / sec / 1e12);   // TFLOP/s
    else if (kind == PEAK_MFMA_VALU) *h_result = (float)(256.0 * 8 * mfma_rounds * 8 * 16384.0 / sec / 1e12);  // TFLOP/s of the MFMAs: 256 blocks of 8 waves
    else *h_result = (float)((kind == PEAK_COPY || kind == PEAK_COPY_NT ? 2.0 : 1.0) * (double)nbytes / sec / 1e9);  // GB/s
    return PPO_OK;
  };
  const int rc = body();
  if (rc) g_create_error = c->err;
  free_all(c);
  return rc;
}

}  // extern "C"
