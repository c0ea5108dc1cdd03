"""Seeded synthetic rollouts and parameter initialisation.

Stands in for the paper's simulator (Algorithm 1), which is not available:
depth images are a 2.0 m background with 1-4 rectangles at U(0.2, 1.5) m,
sigma = 0.01 pixel noise and 5 % zeroed pixels; stereo views are uniform [0,1]
RGB with random coloured rectangles.  This module holds input generation only
(no arithmetic of the learner) and is the one module used by both the HIP
path's harness and the test oracle's harness.

Everything is drawn from numpy's PCG64 with explicit seeds.
"""
from __future__ import annotations

import math

import numpy as np
import torch

from .configs import layer_shapes

_CHUNK = 256


def _rects(rng, n, h, w):
    cnt = rng.integers(1, 5, size=n)
    out = []
    for k in range(4):
        top = rng.integers(0, h, size=n)
        left = rng.integers(0, w, size=n)
        rh = rng.integers(max(1, h // 8), h // 2 + 1, size=n)
        rw = rng.integers(max(1, w // 8), w // 2 + 1, size=n)
        out.append((cnt > k, top, left, rh, rw))
    return out


def _paint(img, rects, values):
    """img [n][c][h][w]; values[k] [n][c]; later rectangles overwrite earlier ones."""
    n, c, h, w = img.shape
    ys = np.arange(h)[None, :, None]
    xs = np.arange(w)[None, None, :]
    for (on, top, left, rh, rw), val in zip(rects, values):
        m = (on[:, None, None] & (ys >= top[:, None, None]) & (ys < (top + rh)[:, None, None])
             & (xs >= left[:, None, None]) & (xs < (left + rw)[:, None, None]))
        img[...] = np.where(m[:, None], val[:, :, None, None], img)
    return img


def depth_images(rng, n, h, w):
    """float32 [n][1][h][w] depth maps in metres (not yet narrowed)."""
    out = np.empty((n, 1, h, w), np.float32)
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        m = b - a
        img = np.full((m, 1, h, w), 2.0, np.float32)
        rects = _rects(rng, m, h, w)
        vals = [rng.uniform(0.2, 1.5, size=(m, 1)).astype(np.float32) for _ in range(4)]
        _paint(img, rects, vals)
        img += 0.01 * rng.standard_normal(img.shape, dtype=np.float32)
        img[rng.random(img.shape, dtype=np.float32) < 0.05] = 0.0
        out[a:b] = img
    return out


def rgb_images(rng, n, h, w):
    """float32 [n][3][h][w], uniform [0,1] texture with 1-4 random coloured rectangles."""
    out = np.empty((n, 3, h, w), np.float32)
    for a in range(0, n, _CHUNK):
        b = min(n, a + _CHUNK)
        m = b - a
        img = rng.random((m, 3, h, w), dtype=np.float32)
        rects = _rects(rng, m, h, w)
        vals = [rng.random((m, 3), dtype=np.float32) for _ in range(4)]
        out[a:b] = _paint(img, rects, vals)
    return out


def narrow_bf16(x: np.ndarray) -> np.ndarray:
    """One round-to-nearest-even cast to bf16, widened back to float32 (torch's cast)."""
    return torch.from_numpy(np.ascontiguousarray(x, np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def rollout_step(cfg: dict, rng) -> dict:
    """One step's slab for all N envs, as float32/uint8 numpy arrays in canonical layout."""
    net, N = cfg["net"], cfg["num_envs"]
    V, Cc, H, W, P, A = net["n_views"], net["in_c"], net["in_h"], net["in_w"], net["proprio_dim"], net["act_dim"]
    if Cc == 1:
        obs = np.stack([depth_images(rng, N, H, W) for _ in range(V)], axis=1)
    else:
        obs = np.stack([rgb_images(rng, N, H, W) for _ in range(V)], axis=1)
    if cfg["obs_dtype"] == "bf16":
        obs = narrow_bf16(obs)
    proprio = rng.standard_normal((N, P), dtype=np.float32)
    action = rng.standard_normal((N, A), dtype=np.float32)
    # behaviour log-prob: unit Gaussian density of the action plus a small perturbation, so that
    # probability ratios fall on both sides of the clip range
    logp = (-0.5 * (action.astype(np.float64) ** 2).sum(1) - 0.5 * A * math.log(2 * math.pi)
            + 0.1 * rng.standard_normal(N)).astype(np.float32)
    value = rng.standard_normal(N, dtype=np.float32)
    reward = rng.standard_normal(N, dtype=np.float32)
    done = (rng.random(N) < 0.01).astype(np.uint8)
    return dict(obs=obs, proprio=proprio, action=action, logp_old=logp, value=value, reward=reward, done=done)


def rollout(cfg: dict, seed: int | None = None, conditioned: bool = False) -> dict:
    """All T steps stacked ([T][N]...), plus last_value [N].

    conditioned=False: the benchmark recipe, every scalar field independent noise.  The batch gradient of
    such a rollout is a sum of B zero-mean terms that cancels like sqrt(B).
    conditioned=True: the same observations, proprioception and actions, but the fields a learner regresses
    on are fixed functions of them, so the batch gradient is a coherent sum (what a real rollout gives):
      PPO:      reward = u.a + 1 + 0.1 eps   (u a fixed unit vector: advantages favour one action direction),
                value  = 0.5 w.proprio + 0.1 eps (w a fixed unit vector), last_value = 0.1 eps;
      student:  teacher action = c + 0.5 M proprio + 0.1 eps  (c in {-1, +1}^A, M fixed with rows of unit
                expected norm), stored in the action slot.
    u, w, c, M come from a generator seeded with seed + 99 only."""
    s0 = cfg["seed"] if seed is None else seed
    rng = np.random.default_rng(s0)
    steps = [rollout_step(cfg, rng) for _ in range(cfg["horizon"])]
    out = {k: np.stack([s[k] for s in steps]) for k in steps[0]}
    out["last_value"] = rng.standard_normal(cfg["num_envs"], dtype=np.float32)
    if conditioned:
        A, P = cfg["net"]["act_dim"], cfg["net"]["proprio_dim"]
        r2 = np.random.default_rng(s0 + 99)
        if cfg["kind"] == "distill":
            c = r2.choice(np.array([-1.0, 1.0], np.float32), A)
            M = (r2.standard_normal((P, A)) / math.sqrt(P)).astype(np.float32)
            out["action"] = (c + 0.5 * (out["proprio"] @ M) + 0.1 * out["action"]).astype(np.float32)
        else:
            u = r2.standard_normal(A).astype(np.float32)
            u /= np.linalg.norm(u)
            w = r2.standard_normal(P).astype(np.float32)
            w /= np.linalg.norm(w)
            out["reward"] = (out["action"] @ u + 1.0 + 0.1 * out["reward"]).astype(np.float32)
            out["value"] = (0.5 * (out["proprio"] @ w) + 0.1 * out["value"]).astype(np.float32)
            out["last_value"] = (0.1 * out["last_value"]).astype(np.float32)
    return out


def param_layout(net: dict):
    """[(name, shape, fan_in)] in canonical order: per conv layer W, b, [layer-norm gain, shift]; [embedding W, b];
    per LSTM layer W_ih, W_hh, b (gates i, f, g, o); per hidden layer W, b; mu W, b; [v w, b, logstd];
    [auxiliary MLP head W1, b1, W2, b2]."""
    shp = layer_shapes(net)
    k = net["conv_k"]
    items = []
    for i, ((ci, _, _), (co, _, _)) in enumerate(zip(shp[:-1], shp[1:])):
        items += [(f"conv{i}.w", (co, ci, k, k), ci * k * k), (f"conv{i}.b", (co,), ci * k * k)]
        if net.get("layer_norm", 0):
            items += [(f"ln{i}.g", (co,), 0), (f"ln{i}.b", (co,), 0)]
    c, h, w = shp[-1]
    enc = c * h * w
    if net.get("embed_dim", 0):
        items += [("emb.w", (net["embed_dim"], enc), enc), ("emb.b", (net["embed_dim"],), enc)]
        enc = net["embed_dim"]
    fin = net["n_views"] * enc + net["proprio_dim"]
    H = net.get("lstm_units", 0)
    for i in range(net.get("lstm_layers", 0)):
        items += [(f"lstm{i}.wih", (4 * H, fin), H), (f"lstm{i}.whh", (4 * H, H), H), (f"lstm{i}.b", (4 * H,), H)]
        fin = H
    for i, f in enumerate(net["fc_dim"]):
        items += [(f"fc{i}.w", (f, fin), fin), (f"fc{i}.b", (f,), fin)]
        fin = f
    A = net["act_dim"]
    X, xh = (net.get("aux_dim", 0), net.get("aux_hidden", 0)) if net.get("aux_hidden", 0) else (0, 0)
    items += [("mu.w", (A - X, fin), fin), ("mu.b", (A - X,), fin)]
    if net["has_value_head"]:
        items += [("v.w", (fin,), fin), ("v.b", (1,), fin), ("logstd", (A,), 0)]
    if xh:
        items += [("aux1.w", (xh, fin), fin), ("aux1.b", (xh,), fin), ("aux2.w", (X, xh), xh), ("aux2.b", (X,), xh)]
    return items


def param_slices(net: dict) -> dict:
    out, off = {}, 0
    for name, shape, _ in param_layout(net):
        n = int(np.prod(shape))
        out[name] = (off, off + n, shape)
        off += n
    return out


def init_params(net: dict, seed: int) -> np.ndarray:
    """Canonical float32 parameter vector: weights and biases U(+-1/sqrt(fan_in)), the action
    head scaled by 0.01, log-std 0."""
    rng = np.random.default_rng(seed + 7919)
    parts = []
    for name, shape, fan_in in param_layout(net):
        if name == "logstd":
            parts.append(np.zeros(shape, np.float32))
            continue
        if name.startswith("ln"):   # gains around 1, small shifts (exactly 1 and 0 would hide a swapped pair)
            parts.append((rng.uniform(0.5, 1.5, size=shape) if name.endswith(".g") else rng.uniform(-0.1, 0.1, size=shape)).astype(np.float32))
            continue
        bound = 1.0 / math.sqrt(fan_in)
        x = rng.uniform(-bound, bound, size=shape).astype(np.float32)
        if name.startswith("mu."):
            x *= 0.01
        parts.append(x)
    return np.concatenate([p.reshape(-1) for p in parts])


# ---------------------------------------------------------------------------------------------
# The same recipe drawn on the GPU with torch's seeded generator: used by the benchmark, where the
# large workloads (up to 10^10 pixels) would take minutes to draw on the host.  Same distributions,
# different random stream than the numpy generators above (which feed the parity tests).
def _rects_torch(gen, n, h, w, dev):
    ri = lambda lo, hi: torch.randint(lo, hi, (n,), generator=gen, device=dev)
    cnt = ri(1, 5)
    return [(cnt > k, ri(0, h), ri(0, w), ri(max(1, h // 8), h // 2 + 1), ri(max(1, w // 8), w // 2 + 1)) for k in range(4)]


def _paint_torch(img, rects, values):
    n, c, h, w = img.shape
    ys = torch.arange(h, device=img.device)[None, :, None]
    xs = torch.arange(w, device=img.device)[None, None, :]
    for (on, top, left, rh, rw), val in zip(rects, values):
        m = (on[:, None, None] & (ys >= top[:, None, None]) & (ys < (top + rh)[:, None, None])
             & (xs >= left[:, None, None]) & (xs < (left + rw)[:, None, None]))
        img = torch.where(m[:, None], val[:, :, None, None], img)
    return img


def rollout_step_torch(cfg: dict, gen, device="cuda") -> dict:
    """One step's slab for all N envs as CUDA tensors (obs already in the config's dtype)."""
    net, N = cfg["net"], cfg["num_envs"]
    V, Cc, H, W, P, A = net["n_views"], net["in_c"], net["in_h"], net["in_w"], net["proprio_dim"], net["act_dim"]
    u = lambda *s: torch.rand(*s, generator=gen, device=device)
    g = lambda *s: torch.randn(*s, generator=gen, device=device)
    views = []
    for _ in range(V):
        chunks = []
        for a in range(0, N, 2048):
            m = min(N, a + 2048) - a
            rects = _rects_torch(gen, m, H, W, device)
            if Cc == 1:
                img = torch.full((m, 1, H, W), 2.0, device=device)
                img = _paint_torch(img, rects, [0.2 + 1.3 * u(m, 1) for _ in range(4)])
                img = img + 0.01 * g(m, 1, H, W)
                img = torch.where(u(m, 1, H, W) < 0.05, torch.zeros_like(img), img)
            else:
                img = _paint_torch(u(m, Cc, H, W), rects, [u(m, Cc) for _ in range(4)])
            chunks.append(img.to(torch.float32 if cfg["obs_dtype"] == "fp32" else torch.bfloat16))
        views.append(torch.cat(chunks))
    obs = torch.stack(views, dim=1).contiguous()
    action = g(N, A)
    logp = (-0.5 * (action.double() ** 2).sum(1) - 0.5 * A * math.log(2 * math.pi) + 0.1 * g(N).double()).float()
    return dict(obs=obs, proprio=g(N, P), action=action, logp_old=logp, value=g(N), reward=g(N),
                done=(u(N) < 0.01).to(torch.uint8))
