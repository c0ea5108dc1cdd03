"""Harness shared by the GPU parity tests: pushes one seeded synthetic rollout through
the library's ppo_buffer_write and hands the same arrays (flattened to s = t*N + n) to
the oracle."""
import numpy as np

from paper_2509_16434_amd import synth

TOL_GAE = 1e-5      # fp32 GAE / returns, relative to max(1, |y|)
TOL_BF16 = 2e-2     # loss scalars, gradients, updated parameters (bf16 MFMA, fp32 accumulate)


def rel_l2(x, y):
    x, y = np.asarray(x, np.float64), np.asarray(y, np.float64)
    return float(np.linalg.norm(x - y) / max(np.linalg.norm(y), 1e-30))


def flat_rollout(ro):
    """[T][N]... -> [S]... with s = t*N + n."""
    T, N = ro["reward"].shape
    out = {k: v.reshape((T * N,) + v.shape[2:]) for k, v in ro.items() if k != "last_value"}
    out["last_value"] = ro["last_value"]
    return out


def fill_learner(lrn, cfg, ro, distill=False):
    import torch
    odt = torch.float32 if cfg["obs_dtype"] == "fp32" else torch.bfloat16
    for t in range(cfg["horizon"]):
        obs = torch.from_numpy(ro["obs"][t]).to("cuda").to(odt).contiguous()
        args = [torch.from_numpy(ro[k][t]).to("cuda").contiguous() for k in ("proprio", "action")]
        if distill:
            lrn.buffer_write(t, obs, *args)
        else:
            extra = [torch.from_numpy(ro[k][t]).to("cuda").contiguous() for k in ("logp_old", "value", "reward", "done")]
            lrn.buffer_write(t, obs, *args, *extra)
    lrn.synchronize()


def per_tensor_errors(net, got, want):
    """{tensor name: relative L2 error} over the canonical parameter layout."""
    return {name: rel_l2(got[a:b], want[a:b]) for name, (a, b, _) in synth.param_slices(net).items()}


def per_tensor_param_errors(net, got, want, steps, lr):
    """Relative L2 error of updated parameters per tensor.  The scale of a tensor is the larger of its
    own norm and sqrt(n)*steps*lr, the farthest Adam can have moved it: a tensor initialised near zero
    (the 0.01-scaled action head) consists almost entirely of Adam steps, whose per-element sign for
    gradient elements below the bf16 noise floor is not determined by the arithmetic being compared."""
    out = {}
    for name, (a, b, _) in synth.param_slices(net).items():
        w = np.asarray(want[a:b], np.float64)
        scale = max(np.linalg.norm(w), np.sqrt(b - a) * steps * lr)
        out[name] = float(np.linalg.norm(np.asarray(got[a:b], np.float64) - w) / scale)
    return out
