"""Workload registry: the five benchmark configurations, and the paper's second resolution, as plain data.

Holds no arithmetic of the method; both the HIP binding and the test oracle
read their network geometry and hyper-parameters from here.  Index = position
in the benchmark's config list (0 tiny, 1 medium, 2 full, 3 stereo
distillation, 4 large batch).  Horizon 16 and the 7+16 = 23-d action space
follow the paper (Sec. III-B sizing example; Sec. III-C robot description);
resolution 160x120 is the paper's Table I row 1.  Index 5 is Table I row 2: 320x240 depth at the
2100 environments the disaggregated set-up reaches there, with the network and hyper-parameters of
the full configuration.  Index 6 is the paper's own teacher (Sec. III-C, Fig. 3: 4-layer CNN [16, 32, 64, 128] with
layer normalisation, 32-d embedding, two LSTM layers of 1024 units, MLP [512, 512, 256]) at the 1024 environments one
GPU of the data-parallel set-up holds at 160x120 (Table I), trained on minibatches of whole environments.
"""
from __future__ import annotations

import copy

_PPO_HP = dict(gamma=0.99, lam=0.95, clip_eps=0.2, vclip_eps=0.0, vf_coef=0.5, ent_coef=0.0,
               lr=3e-4, beta1=0.9, beta2=0.999, adam_eps=1e-8)


def _net(n_views, c, h, w, P, A, conv, fc, value=1, **extra):
    return dict(n_views=n_views, in_c=c, in_h=h, in_w=w, proprio_dim=P, act_dim=A,
                conv_ch=list(conv), conv_k=3, conv_stride=2, conv_pad=1, fc_dim=list(fc),
                has_value_head=value, **extra)


CONFIGS = [
    dict(name="c0_tiny", kind="ppo", num_envs=64, horizon=16, obs_dtype="fp32", seed=1234,
         net=_net(1, 1, 32, 32, 32, 12, (8, 16), (64,)),
         hp=dict(_PPO_HP, epochs=1, minibatches=4)),
    dict(name="c1_medium", kind="ppo", num_envs=1024, horizon=16, obs_dtype="bf16", seed=1235,
         net=_net(1, 1, 64, 64, 64, 23, (32, 64, 64), (256, 128)),
         hp=dict(_PPO_HP, epochs=2, minibatches=4)),
    dict(name="c2_full", kind="ppo", num_envs=4096, horizon=16, obs_dtype="bf16", seed=1236,
         net=_net(1, 1, 120, 160, 64, 23, (32, 64, 64, 128), (512, 256, 128)),
         hp=dict(_PPO_HP, epochs=5, minibatches=4, ent_coef=0.01, vclip_eps=0.2)),
    dict(name="c3_stereo_distill", kind="distill", num_envs=4096, horizon=16, obs_dtype="bf16", seed=1237,
         net=_net(2, 3, 120, 160, 64, 23, (32, 64, 64, 128), (512, 256), value=0),
         hp=dict(_PPO_HP, epochs=1, minibatches=8)),
    dict(name="c4_large", kind="ppo", num_envs=16384, horizon=32, obs_dtype="bf16", seed=1238,
         net=_net(1, 1, 120, 160, 64, 23, (32, 64, 64, 128), (512, 256, 128)),
         hp=dict(_PPO_HP, epochs=5, minibatches=8, ent_coef=0.01, vclip_eps=0.2)),
    dict(name="c5_hires", kind="ppo", num_envs=2100, horizon=16, obs_dtype="bf16", seed=1239,
         net=_net(1, 1, 240, 320, 64, 23, (32, 64, 64, 128), (512, 256, 128)),
         hp=dict(_PPO_HP, epochs=5, minibatches=4, ent_coef=0.01, vclip_eps=0.2)),
    dict(name="c6_paper_teacher", kind="ppo", num_envs=1024, horizon=16, obs_dtype="bf16", seed=1240,
         net=_net(1, 1, 120, 160, 64, 23, (16, 32, 64, 128), (512, 512, 256), layer_norm=1, embed_dim=32, lstm_layers=2, lstm_units=1024),
         hp=dict(_PPO_HP, epochs=5, minibatches=4, ent_coef=0.01, vclip_eps=0.2)),
]


def get_config(idx: int, num_envs: int | None = None, horizon: int | None = None) -> dict:
    """Deep copy of config `idx`, optionally with a reduced env count / horizon (same network)."""
    c = copy.deepcopy(CONFIGS[idx])
    if num_envs is not None:
        c["num_envs"] = int(num_envs)
    if horizon is not None:
        c["horizon"] = int(horizon)
    return c


def conv_out(n: int, k: int = 3, s: int = 2, p: int = 1) -> int:
    return (n + 2 * p - k) // s + 1


def layer_shapes(net: dict):
    """[(C,H,W)] of the image and every conv output."""
    shp = [(net["in_c"], net["in_h"], net["in_w"])]
    for co in net["conv_ch"]:
        _, h, w = shp[-1]
        shp.append((co, conv_out(h, net["conv_k"], net["conv_stride"], net["conv_pad"]),
                    conv_out(w, net["conv_k"], net["conv_stride"], net["conv_pad"])))
    return shp


def param_count(net: dict) -> int:
    shp = layer_shapes(net)
    n = 0
    for (ci, _, _), (co, _, _) in zip(shp[:-1], shp[1:]):
        n += co * ci * net["conv_k"] ** 2 + co + (2 * co if net.get("layer_norm", 0) else 0)
    c, h, w = shp[-1]
    enc = c * h * w
    if net.get("embed_dim", 0):
        n += net["embed_dim"] * enc + net["embed_dim"]
        enc = net["embed_dim"]
    fin = net["n_views"] * enc + net["proprio_dim"]
    for _ in range(net.get("lstm_layers", 0)):
        H = net["lstm_units"]
        n += 4 * H * (fin + H + 1)
        fin = H
    for f in net["fc_dim"]:
        n += fin * f + f
        fin = f
    X, xh = (net.get("aux_dim", 0), net.get("aux_hidden", 0)) if net.get("aux_hidden", 0) else (0, 0)
    n += (net["act_dim"] - X) * (fin + 1)
    if net["has_value_head"]:
        n += fin + 1 + net["act_dim"]
    if xh:
        n += xh * (fin + 1) + X * (xh + 1)
    return n


def flops_per_sample(net: dict) -> dict:
    """Forward and forward+backward FLOPs (2 per multiply-add) of one sample; the
    backward is dgrad + wgrad of every layer except the first conv's dgrad."""
    shp = layer_shapes(net)
    fwd, first = 0, 0
    for i, ((ci, _, _), (co, h, w)) in enumerate(zip(shp[:-1], shp[1:])):
        f = 2 * net["n_views"] * co * h * w * ci * net["conv_k"] ** 2
        fwd += f
        if i == 0:
            first = f
    c, h, w = shp[-1]
    enc = c * h * w
    if net.get("embed_dim", 0):
        fwd += 2 * net["n_views"] * enc * net["embed_dim"]
        enc = net["embed_dim"]
    fin = net["n_views"] * enc + net["proprio_dim"]
    for _ in range(net.get("lstm_layers", 0)):
        fwd += 2 * 4 * net["lstm_units"] * (fin + net["lstm_units"])
        fin = net["lstm_units"]
    for fo in net["fc_dim"]:
        fwd += 2 * fin * fo
        fin = fo
    fwd += 2 * fin * (net["act_dim"] + (1 if net["has_value_head"] else 0))
    if net.get("aux_hidden", 0):
        fwd += 2 * net["aux_hidden"] * (fin + net["aux_dim"])
    return dict(fwd=fwd, fwd_bwd=3 * fwd - first)
