#!/usr/bin/env python3
"""Learner throughput benchmark (one MI355X).

A step is one pass of the whole learner path over one synthetic rollout that is already
resident in HBM: T x ppo_buffer_write, ppo_gae, ppo_update (all epochs x minibatches), or for the
distillation workload T x ppo_buffer_write + distill_update.  The metric is learner
env-steps/s = N*T / time per step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 1] [--no-cpu-baseline] [--phase learn|act]

--phase act times the step in front of the path instead: T x (ppo_act + ppo_buffer_write_outcome), the policy
step of the collection loop on the same observations (metric: policy env-steps/s).

Prints one JSON line.  `roofline` describes the kernel class with the largest share of the step,
timed with HIP events on the library's stream in a second, instrumented pass over the same K steps;
`cpu_baseline` is the CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
PEAK_MFMA_BF16_TF = 2500.0  # dense bf16 MFMA, published
PEAK_FP32_VALU_TF = 157.3   # fp32 vector, published

RIDGE_FLOP_PER_BYTE = PEAK_MFMA_BF16_TF * 1e12 / (PEAK_HBM_GBS * 1e9)  # 312.5

# HBM bytes per launch measured with rocprofv3 counters (FETCH_SIZE and WRITE_SIZE in two runs of this
# script, each scaled by what the same counter reads for the plain copy kernel of ppo_buffer_write in the
# same run: x1.99 and x1.00).  The runs, the raw counter values and the commands are in
# profiles/c1_medium_hbm_traffic.md and profiles/c2_full_hbm_traffic.md; a kernel class or workload that was not
# measured reports null.
MEASURED_TRAFFIC_BYTES = {
    ("c1_medium", "conv_wgrad.1"): 425.9e6,
    ("c1_medium", "conv_fwd.1"): 414.0e6,
    ("c1_medium", "conv_fwd.0"): 320.0e6,
    ("c1_medium", "conv_dgrad.1+wgrad.0"): 184.5e6,
    ("c1_medium", "conv_dgrad.2"): 176.9e6,
    ("c1_medium", "conv_wgrad.2"): 205.0e6,
    ("c1_medium", "conv_fwd.2"): 169.8e6,
    ("c2_full", "conv_fwd.1"): 7900.0e6,
    ("c2_full", "conv_wgrad.1"): 7979.8e6,
    ("c2_full", "conv_fwd.0"): 5982.5e6,
    ("c2_full", "conv_dgrad.1+wgrad.0"): 3642.6e6,
    ("c2_full", "conv_dgrad.2"): 3308.9e6,
    ("c2_full", "conv_fwd.2"): 3282.1e6,
    ("c2_full", "conv_fwd.3"): 1237.5e6,
}


def kernel_bound(rec: dict) -> str:
    """Roofline side of a kernel class: its algorithmic intensity (booked FLOPs / booked bytes) against the
    ridge point of the bf16-MFMA and HBM peaks.  The convolutions of the first layers have K = 9*Cin of a
    few hundred at most and sit on the HBM side; the wide linear layers sit on the MFMA side."""
    if rec["bytes"] <= 0:
        return "mfma"
    return "mfma" if rec["flops"] / rec["bytes"] > RIDGE_FLOP_PER_BYTE else "hbm"


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=1, help="index into the benchmark config list (default 1: medium)")
    ap.add_argument("--num-envs", type=int, default=None, help="override the config's env count (debugging only)")
    ap.add_argument("--max-chunk", type=int, default=0, help="samples per forward/backward pass inside a minibatch (0: the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--phase", choices=["learn", "act"], default="learn", help="learn: the learner path (default); act: the policy step")
    ap.add_argument("--profile-table", action="store_true", help="also print the per-kernel-class table to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "Multi-GPU figures are not produced.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_16434_amd import configs, learner, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    cfg = configs.get_config(args.config, num_envs=args.num_envs)
    net, N, T, hp = cfg["net"], cfg["num_envs"], cfg["horizon"], dict(cfg["hp"], seed=cfg["seed"])
    distill = cfg["kind"] == "distill"
    act = args.phase == "act"
    if act and distill:
        print("bench.py: --phase act needs an actor-critic workload", file=sys.stderr)
        sys.exit(2)
    S = N * T

    # ---- synthetic rollout, drawn per step on the GPU (seeded) and kept resident in HBM
    stream = torch.cuda.Stream()
    lrn = learner.Learner(net, N, T, cfg["obs_dtype"], max_chunk=args.max_chunk, stream=stream)
    lrn.set_params(synth.init_params(net, cfg["seed"]))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg["seed"])
    fl = configs.flops_per_sample(net)
    n_cpu = int(max(8, min(S, 4.0e11 / fl["fwd_bwd"])))  # ~4e11 FLOPs of oracle work, about 10-30 s of CPU time
    steps_dev, host_steps = [], []
    for t in range(T):
        d = synth.rollout_step_torch(cfg, gen)
        if len(host_steps) * N < n_cpu:
            host_steps.append({k: v.float().cpu().numpy() if v.dtype != torch.uint8 else v.cpu().numpy() for k, v in d.items()})
        steps_dev.append(d)
    last_value = torch.randn(N, generator=gen, device="cuda")
    noise = [torch.randn(N, net["act_dim"], generator=gen, device="cuda") for _ in range(T)] if act else None
    torch.cuda.synchronize()

    def one_step():
        if act:
            for t, d in enumerate(steps_dev):
                lrn.act(t, d["obs"], d["proprio"], noise[t])
                lrn.buffer_write_outcome(t, d["reward"], d["done"])
            return
        for t, d in enumerate(steps_dev):
            if distill:
                lrn.buffer_write(t, d["obs"], d["proprio"], d["action"])
            else:
                lrn.buffer_write(t, d["obs"], d["proprio"], d["action"], d["logp_old"], d["value"], d["reward"], d["done"])
        if distill:
            lrn.distill_update(hp, want_stats=False)
        else:
            lrn.gae(last_value, hp["gamma"], hp["lam"])
            lrn.update(hp, want_stats=False)

    for _ in range(args.warmup):
        one_step()
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    stream.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    value = S / (dt / args.steps)

    # ---- instrumented pass: HIP events around every kernel class, same K steps
    lrn.profile(True)
    for _ in range(args.steps):
        one_step()
    rep = lrn.profile_report()
    lrn.profile(False)
    tot_ms = sum(r["ms"] for r in rep.values())
    dom = max(rep, key=lambda k: rep[k]["ms"])
    r = rep[dom]
    avg_s = r["ms"] / r["launches"] * 1e-3
    if kernel_bound(r) == "mfma":
        ach, peak, unit = r["flops"] / r["launches"] / avg_s / 1e12, PEAK_MFMA_BF16_TF, "TFLOP/s"
    else:
        ach, peak, unit = r["bytes"] / r["launches"] / avg_s / 1e9, PEAK_HBM_GBS, "GB/s"
    roofline = dict(bound=kernel_bound(r), kernel=dom, intensity_flop_per_byte=round(r["flops"] / max(r["bytes"], 1.0), 1), achieved=round(ach, 3), peak=peak, unit=unit,
                    frac=round(ach / peak, 5),
                    traffic=MEASURED_TRAFFIC_BYTES.get((cfg["name"], dom)) if args.num_envs is None and not act else None,
                    algorithmic_bytes_per_launch=round(r["bytes"] / r["launches"], 1), avg_launch_us=round(avg_s * 1e6, 2),
                    launches_per_step=r["launches"] / args.steps, share_of_kernel_time=round(r["ms"] / tot_ms, 4))
    step_flops = fl["fwd"] * S if act else fl["fwd_bwd"] * S * hp["epochs"]
    if args.profile_table:
        print(f"{'class':<16}{'launches':>9}{'ms/step':>10}{'share':>8}{'TFLOP/s':>10}{'GB/s':>10}", file=sys.stderr)
        for k in sorted(rep, key=lambda k: -rep[k]["ms"]):
            q = rep[k]
            sec = q["ms"] * 1e-3
            print(f"{k:<16}{q['launches'] // args.steps:>9}{q['ms'] / args.steps:>10.4f}{q['ms'] / tot_ms:>8.3f}"
                  f"{q['flops'] / sec / 1e12 if sec else 0:>10.2f}{q['bytes'] / sec / 1e9 if sec else 0:>10.1f}", file=sys.stderr)
        print(f"kernel time {tot_ms / args.steps:.3f} ms/step vs wall {ms_per_step:.3f} ms/step", file=sys.stderr)

    # ---- CPU oracle on a bounded sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import ppo_oracle as orc
        n_sub = min(n_cpu, len(host_steps) * N)
        sub = {k: np.concatenate([h[k] for h in host_steps])[:n_sub] for k in host_steps[0]}
        p = synth.init_params(net, cfg["seed"])
        t1 = time.perf_counter()
        if act:
            n_sub = min(n_sub * 3, len(host_steps) * N)  # forward only: a third of the work per sample
            sub = {k: v[:n_sub] for k, v in {k: np.concatenate([h[k] for h in host_steps]) for k in host_steps[0]}.items()}
            orc.act(net, p, sub["obs"], sub["proprio"], np.zeros((n_sub, net["act_dim"])))
        elif distill:
            orc.distill_loss_grad(net, p, sub["obs"], sub["proprio"], sub["action"])
        else:
            orc.ppo_loss_grad(net, p, sub["obs"], sub["proprio"], sub["action"], sub["logp_old"], sub["value"],
                              np.zeros(n_sub), np.zeros(n_sub), clip_eps=hp["clip_eps"], vclip_eps=hp["vclip_eps"],
                              vf_coef=hp["vf_coef"], ent_coef=hp["ent_coef"])
        t_mb = time.perf_counter() - t1
        if act:
            cpu = dict(value=round(n_sub / t_mb, 3), unit="env-steps/s", cores=orc.num_threads(), kind="oracle",
                       sample=f"policy step of {n_sub} of the {S} observations timed ({t_mb:.1f} s)")
        # GAE and the permutations at full size (cheap), then extrapolate the network part linearly in samples
        t2 = time.perf_counter()
        if not distill and not act:
            z = np.zeros((T, N))
            orc.gae(z, np.zeros((T, N), np.uint8), z, np.zeros(N), hp["gamma"], hp["lam"])
        for e in range(0 if act else hp["epochs"]):
            orc.permutation(hp["seed"], 0, e, S)
        t_small = time.perf_counter() - t2
        t_full = t_mb / n_sub * S * hp["epochs"] + t_small
        if not act:
          cpu = dict(value=round(S / t_full, 3), unit="env-steps/s", cores=orc.num_threads(), kind="oracle",
                     sample=f"forward+loss+backward of {n_sub} of the {S} samples timed ({t_mb:.1f} s), extrapolated "
                            f"linearly to {hp['epochs']} epochs; GAE and permutations timed at full size")

    out = {
        "metric": "policy env-steps/sec (act + buffer append)" if act else
                  "learner env-steps/sec (GAE + PPO epochs)" if not distill else "learner env-steps/sec (distillation update)",
        "value": round(value, 1), "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg["name"], "num_envs": N, "horizon": T, "obs": f"{net['n_views']}x{net['in_c']}x{net['in_h']}x{net['in_w']} {cfg['obs_dtype']}",
                   "epochs": hp["epochs"], "minibatches": hp["minibatches"], "params": configs.param_count(net)},
        "achieved_tflops": round(step_flops / (dt / args.steps) / 1e12, 3),
        "mfma_frac_of_peak": round(step_flops / (dt / args.steps) / 1e12 / PEAK_MFMA_BF16_TF, 5),
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
