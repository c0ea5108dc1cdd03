"""Thin ctypes binding of libppo_learner.so (see include/ppo_learner.h).

Argument marshalling only: every step of the path runs in the library's HIP
kernels.  PyTorch is used for device memory and the stream, nothing else.  There
is no CPU fallback: if the library is missing or fails to load, importing this
module raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libppo_learner.so")
MAXL = 8

PPO_OK, PPO_EINVAL, PPO_ESHAPE, PPO_ESTATE, PPO_EHIP, PPO_ENOMEM = 0, -1, -2, -3, -4, -5
_ERR = {PPO_EINVAL: "PPO_EINVAL", PPO_ESHAPE: "PPO_ESHAPE", PPO_ESTATE: "PPO_ESTATE", PPO_EHIP: "PPO_EHIP",
        PPO_ENOMEM: "PPO_ENOMEM"}
STAT_FIELDS = ("pi_loss", "v_loss", "entropy", "approx_kl", "clip_frac", "grad_norm", "total_loss")


class NetDesc(C.Structure):
    _fields_ = [("num_envs", C.c_int32), ("horizon", C.c_int32),
                ("n_views", C.c_int32), ("in_c", C.c_int32), ("in_h", C.c_int32), ("in_w", C.c_int32),
                ("obs_dtype", C.c_int32), ("proprio_dim", C.c_int32), ("act_dim", C.c_int32),
                ("n_conv", C.c_int32), ("conv_ch", C.c_int32 * MAXL),
                ("conv_k", C.c_int32), ("conv_stride", C.c_int32), ("conv_pad", C.c_int32),
                ("n_fc", C.c_int32), ("fc_dim", C.c_int32 * MAXL),
                ("has_value_head", C.c_int32), ("max_chunk", C.c_int32),
                ("aux_hidden", C.c_int32), ("aux_dim", C.c_int32),
                ("layer_norm", C.c_int32), ("embed_dim", C.c_int32), ("lstm_layers", C.c_int32), ("lstm_units", C.c_int32)]


class HParams(C.Structure):
    _fields_ = [("gamma", C.c_float), ("lam", C.c_float), ("clip_eps", C.c_float), ("vclip_eps", C.c_float),
                ("vf_coef", C.c_float), ("ent_coef", C.c_float), ("lr", C.c_float), ("beta1", C.c_float),
                ("beta2", C.c_float), ("adam_eps", C.c_float), ("max_grad_norm", C.c_float),
                ("desired_kl", C.c_float), ("lr_min", C.c_float), ("lr_max", C.c_float),
                ("aux_coef", C.c_float),
                ("epochs", C.c_int32), ("minibatches", C.c_int32), ("norm_adv", C.c_int32), ("lr_carry", C.c_int32),
                ("aux_dim", C.c_int32), ("seed", C.c_uint64)]


class MbStats(C.Structure):
    _fields_ = [(f, C.c_float) for f in STAT_FIELDS] + [("nonfinite", C.c_int32), ("lr", C.c_float)]


class LearnerError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"{_ERR.get(code, code)}: {msg}")
        self.code = code


def load_library():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2509_16434_amd/build.py). There is no fallback path.")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u64 = C.c_void_p, C.c_int32, C.c_int64, C.c_uint64
    fp = C.POINTER(C.c_float)
    sig = {
        "ppo_create": (C.c_int, [C.POINTER(vp), C.POINTER(NetDesc), vp]),
        "ppo_destroy": (C.c_int, [vp]),
        "ppo_last_error": (C.c_char_p, [vp]),
        "ppo_param_count": (i64, [vp]),
        "ppo_buffer_image_bytes": (i64, [vp]),
        "ppo_set_params": (C.c_int, [vp, fp, i64]),
        "ppo_get_params": (C.c_int, [vp, fp, i64]),
        "ppo_get_grads": (C.c_int, [vp, fp, i64]),
        "ppo_set_opt_state": (C.c_int, [vp, fp, fp, i64, i64, i64]),
        "ppo_get_opt_state": (C.c_int, [vp, fp, fp, i64, C.POINTER(i64), C.POINTER(i64)]),
        "ppo_get_adaptive_lr": (C.c_int, [vp, fp, C.POINTER(i32)]),
        "ppo_set_adaptive_lr": (C.c_int, [vp, C.c_float, i32]),
        "ppo_buffer_write": (C.c_int, [vp, i32, vp, vp, vp, vp, vp, vp, vp]),
        "ppo_buffer_write_range": (C.c_int, [vp, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp]),
        "ppo_act": (C.c_int, [vp, i32, vp, vp, vp, vp, vp, vp]),
        "ppo_buffer_write_outcome": (C.c_int, [vp, i32, vp, vp]),
        "ppo_buffer_write_state": (C.c_int, [vp, vp, vp]),
        "ppo_buffer_read_obs": (C.c_int, [vp, i32, vp]),
        "ppo_gae": (C.c_int, [vp, vp, C.c_float, C.c_float]),
        "ppo_get_adv_ret": (C.c_int, [vp, vp, vp]),
        "ppo_permutation": (C.c_int, [vp, u64, u64, u64, C.POINTER(i32)]),
        "ppo_permutation_static": (C.c_int, [i64, u64, u64, u64, vp, vp]),
        "ppo_update": (C.c_int, [vp, C.POINTER(HParams), C.POINTER(MbStats)]),
        "distill_update": (C.c_int, [vp, C.POINTER(HParams), C.POINTER(MbStats)]),
        "ppo_forward": (C.c_int, [vp, vp, i64, vp, vp]),
        "ppo_profile": (C.c_int, [vp, i32]),
        "ppo_profile_report": (i64, [vp, C.c_char_p, i64]),
        "ppo_diag_gemm": (C.c_int, [i32, i32, i32, fp, fp, fp]),
        "ppo_diag_peak": (C.c_int, [i32, i64, i32, fp]),
    }
    for name, (res, args) in sig.items():
        f = getattr(lib, name)
        f.restype, f.argtypes = res, args
    return lib


_lib = load_library()
EXPORTS = ("ppo_create", "ppo_destroy", "ppo_last_error", "ppo_param_count", "ppo_buffer_image_bytes",
           "ppo_set_params", "ppo_get_params", "ppo_get_grads", "ppo_set_opt_state", "ppo_get_opt_state", "ppo_get_adaptive_lr", "ppo_set_adaptive_lr",
           "ppo_buffer_write", "ppo_buffer_write_range", "ppo_act", "ppo_buffer_write_outcome", "ppo_buffer_write_state", "ppo_buffer_read_obs", "ppo_gae", "ppo_get_adv_ret", "ppo_permutation", "ppo_permutation_static", "ppo_update", "distill_update",
           "ppo_forward", "ppo_profile", "ppo_profile_report", "ppo_diag_gemm", "ppo_diag_peak")


def make_desc(net: dict, num_envs: int, horizon: int, obs_dtype: str = "bf16", max_chunk: int = 0) -> NetDesc:
    d = NetDesc()
    d.num_envs, d.horizon = num_envs, horizon
    d.n_views, d.in_c, d.in_h, d.in_w = net.get("n_views", 1), net["in_c"], net["in_h"], net["in_w"]
    d.obs_dtype = {"fp32": 0, "bf16": 1}[obs_dtype]
    d.proprio_dim, d.act_dim = net["proprio_dim"], net["act_dim"]
    d.n_conv = len(net["conv_ch"])
    for i, c in enumerate(net["conv_ch"]):
        d.conv_ch[i] = c
    d.conv_k, d.conv_stride, d.conv_pad = net.get("conv_k", 3), net.get("conv_stride", 2), net.get("conv_pad", 1)
    d.n_fc = len(net["fc_dim"])
    for i, c in enumerate(net["fc_dim"]):
        d.fc_dim[i] = c
    d.has_value_head = int(net.get("has_value_head", 1))
    d.max_chunk = max_chunk
    d.aux_hidden = net.get("aux_hidden", 0)
    d.aux_dim = net.get("aux_dim", 0) if d.aux_hidden else 0
    d.layer_norm, d.embed_dim = int(net.get("layer_norm", 0)), net.get("embed_dim", 0)
    d.lstm_layers = net.get("lstm_layers", 0)
    d.lstm_units = net.get("lstm_units", 0) if d.lstm_layers else 0
    return d


def make_hparams(hp: dict) -> HParams:
    h = HParams()
    h.gamma, h.lam = hp.get("gamma", 0.99), hp.get("lam", 0.95)
    h.clip_eps, h.vclip_eps = hp.get("clip_eps", 0.2), hp.get("vclip_eps", 0.0)
    h.vf_coef, h.ent_coef = hp.get("vf_coef", 0.5), hp.get("ent_coef", 0.0)
    h.lr, h.beta1, h.beta2, h.adam_eps = hp.get("lr", 3e-4), hp.get("beta1", 0.9), hp.get("beta2", 0.999), hp.get("adam_eps", 1e-8)
    h.max_grad_norm = hp.get("max_grad_norm", 0.0)
    h.desired_kl, h.lr_min, h.lr_max = hp.get("desired_kl", 0.0), hp.get("lr_min", 1e-5), hp.get("lr_max", 1e-2)
    h.lr_carry = hp.get("lr_carry", 0)
    h.aux_dim, h.aux_coef = hp.get("aux_dim", 0), hp.get("aux_coef", 1.0)
    h.epochs, h.minibatches, h.norm_adv = hp["epochs"], hp["minibatches"], hp.get("norm_adv", 0)
    h.seed = hp.get("seed", 0)
    return h


def _fp(a: np.ndarray):
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _dev(t, dtype=None, numel=None):
    """Device pointer of a contiguous CUDA tensor (None -> NULL)."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError("expected a contiguous CUDA tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"expected dtype {dtype}, got {t.dtype}")
    if numel is not None and t.numel() != numel:
        raise ValueError(f"expected {numel} elements, got {t.numel()}")
    return C.c_void_p(t.data_ptr())


def diag_gemm(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """C = bf16(A) @ bf16(B)^T through the library's MFMA tile kernel (diagnostic)."""
    a, b = np.ascontiguousarray(a, np.float32), np.ascontiguousarray(b, np.float32)
    M, K = a.shape
    N = b.shape[0]
    c = np.empty((M, N), np.float32)
    rc = _lib.ppo_diag_gemm(M, N, K, _fp(a), _fp(b), _fp(c))
    if rc:
        raise LearnerError(rc, _lib.ppo_last_error(None).decode())
    return c


PEAK_KINDS = {"copy": 0, "copy_read_only": 1, "copy_write_only": 2, "copy_nt": 3, "mfma_bf16_loop": 4, "mfma_valu_loop": 5}


def diag_peak(kind: str, nbytes: int = 2 << 30, iters: int = 20) -> float:
    """GB/s (copies; read + written bytes) or TFLOP/s (MFMA loops; for "mfma_valu_loop" nbytes is the number of vector
    instructions per MFMA, 0..8) of a plain kernel on the current GPU (diagnostic)."""
    r = C.c_float()
    rc = _lib.ppo_diag_peak(PEAK_KINDS[kind], nbytes, iters, C.byref(r))
    if rc:
        raise LearnerError(rc, _lib.ppo_last_error(None).decode())
    return float(r.value)


STATIC_PERM_MAX = 1 << 20


def permutation_static(S: int, seed: int, update_idx: int, epoch: int, out=None, stream=None):
    """ppo_permutation_static: the permutation of 0..S-1 into the int32 CUDA tensor `out` (allocated here when
    None; the library itself allocates nothing), enqueued on `stream` (None: the default stream)."""
    import torch
    if out is None:
        out = torch.empty(max(S, 0), dtype=torch.int32, device="cuda")
    sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
    rc = _lib.ppo_permutation_static(S, seed, update_idx, epoch, _dev(out, torch.int32) if S > 0 else None, sp)
    if rc:
        raise LearnerError(rc, _lib.ppo_last_error(None).decode())
    return out


class Learner:
    """One learner context on the current device."""

    def __init__(self, net: dict, num_envs: int, horizon: int, obs_dtype: str = "bf16", max_chunk: int = 0,
                 stream=None):
        import torch
        self._torch = torch
        self.net, self.N, self.T = net, num_envs, horizon
        self.obs_dtype = obs_dtype
        self.desc = make_desc(net, num_envs, horizon, obs_dtype, max_chunk)
        self._h = C.c_void_p()
        self.stream = stream
        sp = C.c_void_p(stream.cuda_stream) if stream is not None else None
        rc = _lib.ppo_create(C.byref(self._h), C.byref(self.desc), sp)
        if rc:
            self._h = C.c_void_p()
            raise LearnerError(rc, _lib.ppo_last_error(None).decode())
        self.n_params = int(_lib.ppo_param_count(self._h))

    # -- plumbing
    def _chk(self, rc):
        if rc:
            raise LearnerError(rc, _lib.ppo_last_error(self._h).decode())

    def close(self):
        if self._h:
            _lib.ppo_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- parameters
    def buffer_image_bytes(self) -> int:
        return int(_lib.ppo_buffer_image_bytes(self._h))

    def set_params(self, p):
        p = np.ascontiguousarray(p, np.float32)
        self._chk(_lib.ppo_set_params(self._h, _fp(p), p.size))

    def get_params(self) -> np.ndarray:
        p = np.empty(self.n_params, np.float32)
        self._chk(_lib.ppo_get_params(self._h, _fp(p), p.size))
        return p

    def get_grads(self) -> np.ndarray:
        p = np.empty(self.n_params, np.float32)
        self._chk(_lib.ppo_get_grads(self._h, _fp(p), p.size))
        return p

    def get_opt_state(self):
        m, v = np.empty(self.n_params, np.float32), np.empty(self.n_params, np.float32)
        step, upd = C.c_int64(), C.c_int64()
        self._chk(_lib.ppo_get_opt_state(self._h, _fp(m), _fp(v), m.size, C.byref(step), C.byref(upd)))
        return m, v, int(step.value), int(upd.value)

    def set_opt_state(self, m, v, step, update_idx):
        m, v = np.ascontiguousarray(m, np.float32), np.ascontiguousarray(v, np.float32)
        self._chk(_lib.ppo_set_opt_state(self._h, _fp(m), _fp(v), m.size, step, update_idx))

    def get_adaptive_lr(self):
        """(rate, live): the KL-adaptive rate carried between updates, live False when there is none."""
        lr, live = C.c_float(), C.c_int32()
        self._chk(_lib.ppo_get_adaptive_lr(self._h, C.byref(lr), C.byref(live)))
        return float(lr.value), bool(live.value)

    def set_adaptive_lr(self, lr: float, live: bool = True):
        self._chk(_lib.ppo_set_adaptive_lr(self._h, lr, int(bool(live))))

    # -- the path
    def buffer_write(self, t, obs, proprio, action, logp=None, value=None, reward=None, done=None):
        torch = self._torch
        net = self.net
        n_obs = self.N * net.get("n_views", 1) * net["in_c"] * net["in_h"] * net["in_w"]
        odt = torch.float32 if self.obs_dtype == "fp32" else torch.bfloat16
        self._chk(_lib.ppo_buffer_write(
            self._h, t, _dev(obs, odt, n_obs), _dev(proprio, torch.float32, self.N * net["proprio_dim"]),
            _dev(action, torch.float32, self.N * net["act_dim"]), _dev(logp, torch.float32, self.N),
            _dev(value, torch.float32, self.N), _dev(reward, torch.float32, self.N), _dev(done, torch.uint8, self.N)))

    def buffer_write_range(self, t, env_offset, obs, proprio, action, logp=None, value=None, reward=None, done=None):
        """Rows [env_offset, env_offset + len(proprio)) of step t."""
        torch, net = self._torch, self.net
        cnt = int(proprio.shape[0])
        n_obs = cnt * net.get("n_views", 1) * net["in_c"] * net["in_h"] * net["in_w"]
        odt = torch.float32 if self.obs_dtype == "fp32" else torch.bfloat16
        self._chk(_lib.ppo_buffer_write_range(
            self._h, t, env_offset, cnt, _dev(obs, odt, n_obs), _dev(proprio, torch.float32, cnt * net["proprio_dim"]),
            _dev(action, torch.float32, cnt * net["act_dim"]), _dev(logp, torch.float32, cnt),
            _dev(value, torch.float32, cnt), _dev(reward, torch.float32, cnt), _dev(done, torch.uint8, cnt)))

    def act(self, t, obs, proprio, noise):
        """Policy step on the step-t observations -> (action [N][A], logp [N], value [N]) device tensors."""
        torch, net = self._torch, self.net
        n_obs = self.N * net.get("n_views", 1) * net["in_c"] * net["in_h"] * net["in_w"]
        odt = torch.float32 if self.obs_dtype == "fp32" else torch.bfloat16
        action = torch.empty(self.N, net["act_dim"], dtype=torch.float32, device="cuda")
        logp = torch.empty(self.N, dtype=torch.float32, device="cuda")
        value = torch.empty(self.N, dtype=torch.float32, device="cuda")
        self._chk(_lib.ppo_act(
            self._h, t, _dev(obs, odt, n_obs), _dev(proprio, torch.float32, self.N * net["proprio_dim"]),
            _dev(noise, torch.float32, self.N * net["act_dim"]), _dev(action), _dev(logp), _dev(value)))
        return action, logp, value

    def buffer_write_outcome(self, t, reward, done):
        torch = self._torch
        self._chk(_lib.ppo_buffer_write_outcome(self._h, t, _dev(reward, torch.float32, self.N), _dev(done, torch.uint8, self.N)))

    def buffer_write_state(self, h0=None, c0=None):
        """Recurrent nets: LSTM state of every environment at the start of the rollout, [layers][N][units] fp32 (None: zeros)."""
        torch, net = self._torch, self.net
        n = net.get("lstm_layers", 0) * self.N * net.get("lstm_units", 0)
        self._chk(_lib.ppo_buffer_write_state(self._h, _dev(h0, torch.float32, n), _dev(c0, torch.float32, n)))

    def buffer_read_obs(self, t):
        torch, net = self._torch, self.net
        out = torch.empty(self.N, net.get("n_views", 1), net["in_c"], net["in_h"], net["in_w"], dtype=torch.bfloat16,
                          device="cuda")
        self._chk(_lib.ppo_buffer_read_obs(self._h, t, _dev(out)))
        self.synchronize()
        return out

    def gae(self, last_value, gamma, lam):
        self._chk(_lib.ppo_gae(self._h, _dev(last_value, self._torch.float32, self.N), gamma, lam))

    def get_adv_ret(self):
        torch = self._torch
        adv = torch.empty(self.T, self.N, dtype=torch.float32, device="cuda")
        ret = torch.empty_like(adv)
        self._chk(_lib.ppo_get_adv_ret(self._h, _dev(adv), _dev(ret)))
        self.synchronize()
        return adv, ret

    def permutation(self, seed, update_idx, epoch) -> np.ndarray:
        out = np.empty(self.N * self.T, np.int32)
        self._chk(_lib.ppo_permutation(self._h, seed, update_idx, epoch, out.ctypes.data_as(C.POINTER(C.c_int32))))
        return out[:self.N] if self.net.get("lstm_layers", 0) else out   # a recurrent net shuffles whole environments

    def _run(self, fn, hp: dict, want_stats: bool):
        h = make_hparams(hp)
        if not want_stats:
            self._chk(fn(self._h, C.byref(h), None))
            return None
        n = hp["epochs"] * hp["minibatches"]
        st = (MbStats * n)()
        self._chk(fn(self._h, C.byref(h), st))
        return [dict({f: float(getattr(s, f)) for f in STAT_FIELDS}, nonfinite=int(s.nonfinite), lr=float(s.lr)) for s in st]

    def update(self, hp: dict, want_stats: bool = True):
        return self._run(_lib.ppo_update, hp, want_stats)

    def distill_update(self, hp: dict, want_stats: bool = True):
        return self._run(_lib.distill_update, hp, want_stats)

    def forward(self, idx=None, count=None):
        torch = self._torch
        if idx is not None:
            count = idx.numel()
        elif count is None:
            count = self.N * self.T
        mu = torch.empty(count, self.net["act_dim"], dtype=torch.float32, device="cuda")
        v = torch.empty(count, dtype=torch.float32, device="cuda") if self.net.get("has_value_head", 1) else None
        self._chk(_lib.ppo_forward(self._h, _dev(idx, torch.int32), count, _dev(mu), _dev(v)))
        self.synchronize()
        return mu, v

    def profile(self, enable: bool):
        self._chk(_lib.ppo_profile(self._h, int(bool(enable))))

    def profile_report(self) -> dict:
        """{class: dict(launches, ms, flops, bytes)} since profile(True)."""
        buf = C.create_string_buffer(1 << 16)
        n = _lib.ppo_profile_report(self._h, buf, len(buf))
        if n < 0:
            self._chk(int(n))
        out = {}
        for line in buf.value.decode().splitlines():
            name, cnt, ms, fl, by = line.split()
            out[name] = dict(launches=int(cnt), ms=float(ms), flops=float(fl), bytes=float(by))
        return out

    def synchronize(self):
        if self.stream is not None:
            self.stream.synchronize()
        else:
            self._torch.cuda.synchronize()
