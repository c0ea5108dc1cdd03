"""ctypes front end of the CPU oracle (oracle/ppo_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The product path (paper_2509_16434_amd) never
imports this module and shares no code with it.

All floating-point arguments are converted to float64 before the C code sees
them; observations stay float32 (bf16 and fp32 images widen exactly).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppo_oracle.c")
_LIB = os.path.join(_HERE, "libppo_oracle.so")
ST_NAMES = ("pi_loss", "v_loss", "entropy", "approx_kl", "clip_frac", "grad_norm", "total", "lr")
ST_N = len(ST_NAMES)
MAXL = 8


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over samples)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Net(C.Structure):
    _fields_ = [("n_views", C.c_int32), ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("proprio_dim", C.c_int32), ("act_dim", C.c_int32),
                ("n_conv", C.c_int32), ("conv_ch", C.c_int32 * MAXL), ("conv_k", C.c_int32),
                ("conv_stride", C.c_int32), ("conv_pad", C.c_int32),
                ("n_fc", C.c_int32), ("fc_dim", C.c_int32 * MAXL), ("has_value_head", C.c_int32),
                ("aux_hidden", C.c_int32), ("aux_dim", C.c_int32),
                ("layer_norm", C.c_int32), ("embed_dim", C.c_int32), ("lstm_layers", C.c_int32), ("lstm_units", C.c_int32)]


class _LossCfg(C.Structure):
    _fields_ = [("clip_eps", C.c_double), ("vclip_eps", C.c_double), ("vf_coef", C.c_double),
                ("ent_coef", C.c_double), ("aux_coef", C.c_double), ("aux_dim", C.c_int32)]


class _AdamCfg(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("max_grad_norm", C.c_double), ("desired_kl", C.c_double), ("lr_min", C.c_double),
                ("lr_max", C.c_double)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_param_count.restype = C.c_int64
        _lib.orc_flat_dim.restype = C.c_int32
        _lib.orc_buffer_image_bytes.restype = C.c_int64
        _lib.orc_buffer_image_bytes.argtypes = [C.c_int64] * 7
        _lib.orc_bf16_rne.restype = C.c_float
        _lib.orc_bf16_rne.argtypes = [C.c_float]
        _lib.orc_splitmix64_nth.restype = C.c_uint64
        _lib.orc_splitmix64_nth.argtypes = [C.c_uint64, C.c_uint64]
        _lib.orc_perm_key.restype = C.c_uint64
        _lib.orc_perm_key.argtypes = [C.c_uint64] * 4
        _lib.orc_num_threads.restype = C.c_int32
    return _lib


def _net(net: dict) -> _Net:
    n = _Net()
    n.n_views = net.get("n_views", 1)
    n.in_c, n.in_h, n.in_w = net["in_c"], net["in_h"], net["in_w"]
    n.proprio_dim, n.act_dim = net["proprio_dim"], net["act_dim"]
    n.n_conv = len(net["conv_ch"])
    for i, c in enumerate(net["conv_ch"]):
        n.conv_ch[i] = c
    n.conv_k, n.conv_stride, n.conv_pad = net.get("conv_k", 3), net.get("conv_stride", 2), net.get("conv_pad", 1)
    n.n_fc = len(net["fc_dim"])
    for i, c in enumerate(net["fc_dim"]):
        n.fc_dim[i] = c
    n.has_value_head = int(net.get("has_value_head", 1))
    n.aux_hidden, n.aux_dim = net.get("aux_hidden", 0), net.get("aux_dim", 0) if net.get("aux_hidden", 0) else 0
    n.layer_norm, n.embed_dim = int(net.get("layer_norm", 0)), net.get("embed_dim", 0)
    n.lstm_layers, n.lstm_units = net.get("lstm_layers", 0), net.get("lstm_units", 0) if net.get("lstm_layers", 0) else 0
    return n


def _d(x):
    return np.ascontiguousarray(x, dtype=np.float64)


def _p(a, t=C.c_double):
    return None if a is None else a.ctypes.data_as(C.POINTER(t))


def param_count(net: dict) -> int:
    n = _net(net)
    return int(lib().orc_param_count(C.byref(n)))


def flat_dim(net: dict) -> int:
    n = _net(net)
    return int(lib().orc_flat_dim(C.byref(n)))


def buffer_image_bytes(N, T, n_views, c, h, w, elem_bytes) -> int:
    return int(lib().orc_buffer_image_bytes(N, T, n_views, c, h, w, elem_bytes))


def bf16_rne(x: np.ndarray) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    out = np.empty_like(x)
    f = lib().orc_bf16_rne
    xf, of = x.reshape(-1), out.reshape(-1)
    for i in range(xf.size):
        of[i] = f(float(xf[i]))
    return out


def gae(reward, done, value, last_value, gamma, lam):
    """reward/done/value [T][N], last_value [N] -> (adv, ret) float64 [T][N]."""
    reward, value, last_value = _d(reward), _d(value), _d(last_value)
    done = np.ascontiguousarray(done, dtype=np.uint8)
    T, N = reward.shape
    adv, ret = np.empty((T, N)), np.empty((T, N))
    lib().orc_gae(C.c_int32(T), C.c_int32(N), _p(reward), _p(done, C.c_uint8), _p(value), _p(last_value),
                  C.c_double(gamma), C.c_double(lam), _p(adv), _p(ret))
    return adv, ret


def splitmix64_nth(state: int, n: int) -> int:
    return int(lib().orc_splitmix64_nth(state, n))


def perm_key(seed: int, update: int, epoch: int, i: int) -> int:
    return int(lib().orc_perm_key(seed, update, epoch, i))


def permutation(seed: int, update: int, epoch: int, S: int) -> np.ndarray:
    out = np.empty(S, dtype=np.int32)
    lib().orc_permutation(C.c_uint64(seed), C.c_uint64(update), C.c_uint64(epoch), C.c_int64(S),
                          _p(out, C.c_int32))
    return out


def _obs(net, obs, B):
    obs = np.ascontiguousarray(obs, dtype=np.float32)
    want = B * net.get("n_views", 1) * net["in_c"] * net["in_h"] * net["in_w"]
    assert obs.size == want, (obs.shape, want)
    return obs


def forward(net, params, obs, proprio):
    """-> mu [B][A], v [B] (zeros without a value head)."""
    n = _net(net)
    proprio = _d(proprio)
    B = proprio.shape[0]
    obs, params = _obs(net, obs, B), _d(params)
    assert params.size == param_count(net)
    mu, v = np.empty((B, net["act_dim"])), np.zeros(B)
    lib().orc_forward(C.byref(n), _p(params), C.c_int64(B), _p(obs, C.c_float), _p(proprio), _p(mu), _p(v))
    return mu, v


def _seq_args(net, proprio, done, h0, c0):
    """Checks the time-major sequence arrays of a recurrent net and returns (L, Benv, done, h0, c0) as C-ready arrays."""
    L, Benv = proprio.shape[0], proprio.shape[1]
    nl, H = net.get("lstm_layers", 0), net.get("lstm_units", 0)
    if done is not None:
        done = np.ascontiguousarray(done, dtype=np.uint8)
        assert done.shape == (L, Benv)
    if h0 is not None:
        h0 = _d(h0)
        assert h0.shape == (nl, Benv, H)
    if c0 is not None:
        c0 = _d(c0)
        assert c0.shape == (nl, Benv, H)
    return L, Benv, done, h0, c0


def seq_forward(net, params, obs, proprio, done=None, h0=None, c0=None):
    """Time-major sequences: obs [L][Benv]..., proprio [L][Benv][P], done [L][Benv], h0/c0 [layers][Benv][H]
    -> mu [L][Benv][A], v [L][Benv], hT, cT [layers][Benv][H]."""
    n = _net(net)
    proprio = _d(proprio)
    L, Benv, done, h0, c0 = _seq_args(net, proprio, done, h0, c0)
    obs, params = _obs(net, obs, L * Benv), _d(params)
    assert params.size == param_count(net)
    nl, H = net.get("lstm_layers", 0), net.get("lstm_units", 0)
    mu, v = np.empty((L, Benv, net["act_dim"])), np.zeros((L, Benv))
    hT, cT = np.zeros((nl, Benv, H)), np.zeros((nl, Benv, H))
    lib().orc_seq_forward(C.byref(n), _p(params), C.c_int64(Benv), C.c_int32(L), _p(obs, C.c_float), _p(proprio),
                          _p(done, C.c_uint8), _p(h0), _p(c0), _p(mu), _p(v), _p(hT), _p(cT))
    return mu, v, hT, cT


def seq_ppo_loss_grad(net, params, obs, proprio, action, logp_old, v_old, adv, ret, done=None, h0=None, c0=None,
                      clip_eps=0.2, vclip_eps=0.0, vf_coef=0.5, ent_coef=0.0):
    """One minibatch of whole sequences (time-major [L][Benv]... arrays) -> (stats, grads)."""
    n = _net(net)
    params, proprio, action = _d(params), _d(proprio), _d(action)
    logp_old, v_old, adv, ret = _d(logp_old), _d(v_old), _d(adv), _d(ret)
    L, Benv, done, h0, c0 = _seq_args(net, proprio, done, h0, c0)
    obs = _obs(net, obs, L * Benv)
    cfg = _LossCfg(clip_eps, vclip_eps, vf_coef, ent_coef)
    grads, st = np.zeros(params.size), np.zeros(ST_N)
    lib().orc_seq_ppo_loss_grad(C.byref(n), _p(params), C.c_int64(Benv), C.c_int32(L), _p(obs, C.c_float), _p(proprio),
                                _p(action), _p(logp_old), _p(v_old), _p(adv), _p(ret), _p(done, C.c_uint8), _p(h0), _p(c0),
                                C.byref(cfg), _p(grads), _p(st))
    return _stats(st), grads


def seq_ppo_update(net, params, m, v, step, obs, proprio, action, logp_old, v_old, adv, ret, hp, done=None, h0=None,
                   c0=None, update_idx=0):
    """Whole PPO update on a rollout given as [T][N] arrays; for a recurrent net the minibatches are whole
    environments (h0/c0 [layers][N][H] are the states at the rollout's start, done flags reset the state)."""
    n = _net(net)
    params, m, v = _d(params).copy(), _d(m).copy(), _d(v).copy()
    proprio, action = _d(proprio), _d(action)
    logp_old, v_old, ret = _d(logp_old), _d(v_old), _d(ret)
    adv = normalize_adv(adv) if hp.get("norm_adv", 0) else _d(adv)
    T, N, done, h0, c0 = _seq_args(net, proprio, done, h0, c0)
    obs = _obs(net, obs, T * N)
    E, M = hp["epochs"], hp["minibatches"]
    assert (N if net.get("lstm_layers", 0) else N * T) % M == 0
    st, gl, stp = np.zeros((E * M, ST_N)), np.zeros(params.size), C.c_int64(step)
    ac = _AdamCfg(hp.get("lr", 3e-4), hp.get("beta1", 0.9), hp.get("beta2", 0.999), hp.get("adam_eps", 1e-8),
                  hp.get("max_grad_norm", 0.0), hp.get("desired_kl", 0.0), hp.get("lr_min", 1e-5), hp.get("lr_max", 1e-2))
    lc = _LossCfg(hp.get("clip_eps", 0.2), hp.get("vclip_eps", 0.0), hp.get("vf_coef", 0.5), hp.get("ent_coef", 0.0))
    lib().orc_seq_ppo_update(C.byref(n), _p(params), _p(m), _p(v), C.byref(stp), C.c_int64(N), C.c_int32(T), _p(obs, C.c_float),
                             _p(proprio), _p(action), _p(logp_old), _p(v_old), _p(adv), _p(ret), _p(done, C.c_uint8), _p(h0),
                             _p(c0), C.byref(lc), C.byref(ac), C.c_int32(E), C.c_int32(M), C.c_uint64(hp.get("seed", 0)),
                             C.c_uint64(update_idx), _p(st), _p(gl))
    return dict(params=params, m=m, v=v, step=int(stp.value), stats=[_stats(r) for r in st], grads_last=gl)


def act(net, params, obs, proprio, noise):
    """Policy step -> action [B][A], logp [B], value [B] (feed-forward actor-critic nets only)."""
    assert net.get("has_value_head", 1) and not net.get("lstm_layers", 0)
    n = _net(net)
    proprio, noise = _d(proprio), _d(noise)
    B = proprio.shape[0]
    obs, params = _obs(net, obs, B), _d(params)
    assert params.size == param_count(net) and noise.shape == (B, net["act_dim"])
    action, logp, value = np.empty((B, net["act_dim"])), np.empty(B), np.empty(B)
    lib().orc_act(C.byref(n), _p(params), C.c_int64(B), _p(obs, C.c_float), _p(proprio), _p(noise), _p(action),
                  _p(logp), _p(value))
    return action, logp, value


def _stats(a):
    return dict(zip(ST_NAMES, (float(x) for x in a)))


def ppo_loss(mu, v, logstd, action, logp_old, v_old, adv, ret, clip_eps=0.2, vclip_eps=0.0,
             vf_coef=0.5, ent_coef=0.0, want_grads=True):
    """Loss on network outputs -> (stats, dmu, dv, dlogstd)."""
    mu, v, logstd, action = _d(mu), _d(v), _d(logstd), _d(action)
    logp_old, v_old, adv, ret = _d(logp_old), _d(v_old), _d(adv), _d(ret)
    B, A = mu.shape
    cfg = _LossCfg(clip_eps, vclip_eps, vf_coef, ent_coef)
    st = np.zeros(ST_N)
    dmu, dv, dls = np.zeros((B, A)), np.zeros(B), np.zeros(A)
    lib().orc_ppo_loss(C.c_int64(B), C.c_int32(A), _p(mu), _p(v), _p(logstd), _p(action), _p(logp_old),
                       _p(v_old), _p(adv), _p(ret), C.byref(cfg), _p(st),
                       _p(dmu) if want_grads else None, _p(dv) if want_grads else None,
                       _p(dls) if want_grads else None)
    return _stats(st), dmu, dv, dls


def mse_loss(pred, target, aux_dim=0, aux_coef=1.0):
    """Distillation loss -> (stats, dpred).  aux_dim > 0: the last aux_dim columns are an auxiliary output whose
    mean squared error (stats["v_loss"]) enters with weight aux_coef beside that of the others (stats["pi_loss"])."""
    pred, target = _d(pred), _d(target)
    B, A = pred.shape
    assert 0 <= aux_dim < A
    st, dp = np.zeros(ST_N), np.zeros((B, A))
    lib().orc_mse_loss(C.c_int64(B), C.c_int32(A), C.c_int32(aux_dim), C.c_double(aux_coef), _p(pred), _p(target),
                       _p(st), _p(dp))
    return _stats(st), dp


def ppo_loss_grad(net, params, obs, proprio, action, logp_old, v_old, adv, ret, clip_eps=0.2,
                  vclip_eps=0.0, vf_coef=0.5, ent_coef=0.0):
    """-> (stats, grads[param_count]) of the PPO objective on one minibatch."""
    n = _net(net)
    params, proprio, action = _d(params), _d(proprio), _d(action)
    logp_old, v_old, adv, ret = _d(logp_old), _d(v_old), _d(adv), _d(ret)
    B = proprio.shape[0]
    obs = _obs(net, obs, B)
    cfg = _LossCfg(clip_eps, vclip_eps, vf_coef, ent_coef)
    grads, st = np.zeros(params.size), np.zeros(ST_N)
    lib().orc_ppo_loss_grad(C.byref(n), _p(params), C.c_int64(B), _p(obs, C.c_float), _p(proprio), _p(action),
                            _p(logp_old), _p(v_old), _p(adv), _p(ret), C.byref(cfg), _p(grads), _p(st))
    return _stats(st), grads


def distill_loss_grad(net, params, obs, proprio, teacher, aux_dim=0, aux_coef=1.0):
    n = _net(net)
    params, proprio, teacher = _d(params), _d(proprio), _d(teacher)
    B = proprio.shape[0]
    obs = _obs(net, obs, B)
    grads, st = np.zeros(params.size), np.zeros(ST_N)
    lib().orc_distill_loss_grad(C.byref(n), _p(params), C.c_int64(B), _p(obs, C.c_float), _p(proprio),
                                _p(teacher), C.c_int32(aux_dim), C.c_double(aux_coef), _p(grads), _p(st))
    return _stats(st), grads


def adam_step(params, m, v, grads, k, lr=3e-4, beta1=0.9, beta2=0.999, eps=1e-8):
    """In-place on float64 arrays params, m, v."""
    for a in (params, m, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    grads = _d(grads)
    cfg = _AdamCfg(lr, beta1, beta2, eps, 0.0)
    lib().orc_adam_step(C.c_int64(params.size), _p(params), _p(m), _p(v), _p(grads), C.c_int64(k), C.byref(cfg))


def clip_grad_norm(grads, max_norm):
    """-> (clipped copy of grads, norm before clipping)."""
    g = _d(grads).copy()
    f = lib().orc_clip_grad_norm
    f.restype = C.c_double
    norm = f(C.c_int64(g.size), _p(g), C.c_double(max_norm))
    return g, float(norm)


def normalize_adv(adv):
    """(adv - mean) / (population std + 1e-8) over all samples."""
    a = _d(adv)
    out = np.empty_like(a)
    lib().orc_normalize_adv(C.c_int64(a.size), _p(a), _p(out))
    return out


def _update(fn_name, net, params, m, v, step, obs, proprio, action, extra, hp, update_idx):
    n = _net(net)
    params, m, v = _d(params).copy(), _d(m).copy(), _d(v).copy()
    proprio, action = _d(proprio), _d(action)
    S = proprio.shape[0]
    obs = _obs(net, obs, S)
    E, M = hp["epochs"], hp["minibatches"]
    assert S % M == 0
    st = np.zeros((E * M, ST_N))
    gl = np.zeros(params.size)
    stp = C.c_int64(step)
    ac = _AdamCfg(hp.get("lr", 3e-4), hp.get("beta1", 0.9), hp.get("beta2", 0.999), hp.get("adam_eps", 1e-8),
                  hp.get("max_grad_norm", 0.0), hp.get("desired_kl", 0.0), hp.get("lr_min", 1e-5),
                  hp.get("lr_max", 1e-2))
    if fn_name == "ppo":
        logp_old, v_old, adv, ret = (_d(x) for x in extra)
        lc = _LossCfg(hp.get("clip_eps", 0.2), hp.get("vclip_eps", 0.0), hp.get("vf_coef", 0.5),
                      hp.get("ent_coef", 0.0))
        lib().orc_ppo_update(C.byref(n), _p(params), _p(m), _p(v), C.byref(stp), C.c_int64(S),
                             _p(obs, C.c_float), _p(proprio), _p(action), _p(logp_old), _p(v_old), _p(adv),
                             _p(ret), C.byref(lc), C.byref(ac), C.c_int32(E), C.c_int32(M),
                             C.c_uint64(hp.get("seed", 0)), C.c_uint64(update_idx), _p(st), _p(gl))
    else:
        lib().orc_distill_update(C.byref(n), _p(params), _p(m), _p(v), C.byref(stp), C.c_int64(S),
                                 _p(obs, C.c_float), _p(proprio), _p(action), C.c_int32(hp.get("aux_dim", 0)),
                                 C.c_double(hp.get("aux_coef", 1.0)), C.byref(ac), C.c_int32(E),
                                 C.c_int32(M), C.c_uint64(hp.get("seed", 0)), C.c_uint64(update_idx),
                                 _p(st), _p(gl))
    return dict(params=params, m=m, v=v, step=int(stp.value), stats=[_stats(r) for r in st], grads_last=gl)


def ppo_update(net, params, m, v, step, obs, proprio, action, logp_old, v_old, adv, ret, hp, update_idx=0):
    """Whole PPO update over flat samples s = t*N + n.  Returns new params/m/v/step, stats, last grads.
    hp["norm_adv"]: advantages normalised over the whole rollout first; hp["max_grad_norm"] > 0: global
    gradient-norm clipping before every Adam step; hp["desired_kl"] > 0: KL-adaptive learning rate between
    hp["lr_min"] and hp["lr_max"], starting from hp["lr"] (stats[i]["lr"] is the rate step i used)."""
    if hp.get("norm_adv", 0):
        adv = normalize_adv(adv)
    return _update("ppo", net, params, m, v, step, obs, proprio, action, (logp_old, v_old, adv, ret), hp,
                   update_idx)


def distill_update(net, params, m, v, step, obs, proprio, teacher, hp, update_idx=0):
    return _update("distill", net, params, m, v, step, obs, proprio, teacher, None, hp, update_idx)


def set_quant(mode: int) -> None:
    """0: exact fp64 (the definition); 1: bf16 operands (stored activations, activation gradients
    and MFMA-layer weights rounded to bf16, wide accumulation)."""
    lib().orc_set_quant(C.c_int32(int(mode)))


def get_quant() -> int:
    return int(lib().orc_get_quant())


class quant:
    """Context manager: `with quant(1): ...`."""

    def __init__(self, mode):
        self.mode = mode

    def __enter__(self):
        self.prev = get_quant()
        set_quant(self.mode)

    def __exit__(self, *a):
        set_quant(self.prev)


def num_threads() -> int:
    return int(lib().orc_num_threads())


def set_num_threads(n: int) -> None:
    lib().orc_set_num_threads(C.c_int32(int(n)))
