#!/usr/bin/env python3
"""Learner throughput benchmark (one MI355X).

A step is one pass of the whole learner path over one synthetic rollout that is already
resident in HBM: T x ppo_buffer_write, ppo_gae, ppo_update (all epochs x minibatches), or for the
distillation workload T x ppo_buffer_write + distill_update.  The metric is learner
env-steps/s = N*T / time per step.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline] [--no-per-config]
                    [--phase learn|act|peaks]

The headline line is the largest single-GPU workload (config 4, c4_large: 16384 envs x 32 steps, a 20 GB
buffer).  The same JSON line carries
  roofline      the kernel class with the largest share of the step, timed with HIP events on the library's
                stream in a second, instrumented pass over the same K steps: HBM side on the kernel's own
                algorithmic bytes; `mfma` beside it prices the same launches by their FLOPs; `traffic` is the
                HBM byte count per launch that rocprofv3 counters measured for that kernel on this workload,
                read from profiles/<workload>_hbm_traffic.md (a tracked summary, not measured by this run);
  phases        achieved GB/s of the HBM-bound side kernels (buffer write, GAE, Adam, permutation) and the
                separate timing of T x ppo_buffer_write;
  per_config    the other workloads (ms/step, env-steps/s, dominant kernel and its fractions), each on a few
                steps of its own;
  cpu_baseline  the CPU oracle on a bounded sample of the headline workload, all host cores and one thread.
--phase act times the step in front of the path instead: T x (ppo_act + ppo_buffer_write_outcome).
--phase peaks measures what plain kernels reach on this GPU (streaming copy / read / write, an MFMA loop).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, published
PEAK_MFMA_BF16_TF = 2500.0  # dense bf16 MFMA, published
PEAK_FP32_VALU_TF = 157.3   # fp32 vector, published

RIDGE_FLOP_PER_BYTE = PEAK_MFMA_BF16_TF * 1e12 / (PEAK_HBM_GBS * 1e9)  # 312.5
HBM_SIDE_CLASSES = ("buffer_write", "gae", "adam", "permutation", "adv_normalize", "wgrad_reduce", "weight_repack")
PER_CONFIG_STEPS = {0: 20, 1: 20, 2: 4, 3: 4, 4: 3, 5: 2, 6: 3}


def kernel_bound(rec: dict) -> str:
    """Roofline side of a kernel class: its algorithmic intensity (booked FLOPs / booked bytes) against the
    ridge point of the bf16-MFMA and HBM peaks.  The convolutions of the first layers have K = 9*Cin of a
    few hundred at most and sit on the HBM side; the wide linear layers sit on the MFMA side."""
    if rec["bytes"] <= 0:
        return "mfma"
    return "mfma" if rec["flops"] / rec["bytes"] > RIDGE_FLOP_PER_BYTE else "hbm"


def measured_traffic(workload: str, klass: str):
    """HBM bytes per launch of kernel class `klass` on `workload` as measured with rocprofv3 counters
    (FETCH_SIZE and WRITE_SIZE, each scaled by the same counter's reading of the plain copy kernel of
    ppo_buffer_write in the same run), read from the table in profiles/<workload>_hbm_traffic.md.
    None when that summary or that row does not exist."""
    path = os.path.join(ROOT, "profiles", f"{workload}_hbm_traffic.md")
    if not os.path.exists(path):
        return None
    col = None
    for line in open(path):
        cells = [c.strip() for c in line.strip().strip("|").split("|")]
        if len(cells) < 4:
            continue
        if "scaled traffic MB" in cells:
            col = (cells.index("class(es)") if "class(es)" in cells else cells.index("class"), cells.index("scaled traffic MB"))
            continue
        if col and klass in [c.strip() for c in cells[col[0]].split(",")]:
            try:
                return float(cells[col[1]]) * 1e6
            except ValueError:
                return None
    return None


def measured_peaks():
    """{name: value} from profiles/peaks.md (what plain kernels reach on the box), or {}."""
    path = os.path.join(ROOT, "profiles", "peaks.md")
    out = {}
    if os.path.exists(path):
        for line in open(path):
            m = re.match(r"\|\s*`?(\w+)`?\s*\|\s*([\d.]+)\s*\|\s*(GB/s|TFLOP/s)\s*\|", line)
            if m:
                out[m.group(1)] = float(m.group(2))
    return out


def roofline_of(rep: dict, workload: str, steps: int, use_traffic: bool) -> dict:
    tot_ms = sum(r["ms"] for r in rep.values())
    dom = max(rep, key=lambda k: rep[k]["ms"])
    r = rep[dom]
    avg_s = r["ms"] / r["launches"] * 1e-3
    gbs = r["bytes"] / r["launches"] / avg_s / 1e9
    tfs = r["flops"] / r["launches"] / avg_s / 1e12
    bound = kernel_bound(r)
    ach, peak, unit = (tfs, PEAK_MFMA_BF16_TF, "TFLOP/s") if bound == "mfma" else (gbs, PEAK_HBM_GBS, "GB/s")
    pk = measured_peaks()
    out = dict(bound=bound, kernel=dom, intensity_flop_per_byte=round(r["flops"] / max(r["bytes"], 1.0), 1),
               achieved=round(ach, 3), peak=peak, unit=unit, frac=round(ach / peak, 5),
               traffic=measured_traffic(workload, dom) if use_traffic else None,
               traffic_source=f"profiles/{workload}_hbm_traffic.md (rocprofv3 counters, not this run)" if use_traffic else None,
               algorithmic_bytes_per_launch=round(r["bytes"] / r["launches"], 1), avg_launch_us=round(avg_s * 1e6, 2),
               launches_per_step=r["launches"] / steps, share_of_kernel_time=round(r["ms"] / tot_ms, 4),
               hbm=dict(achieved=round(gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s", frac=round(gbs / PEAK_HBM_GBS, 5)),
               mfma=dict(achieved=round(tfs, 2), peak=PEAK_MFMA_BF16_TF, unit="TFLOP/s", frac=round(tfs / PEAK_MFMA_BF16_TF, 5)))
    if pk.get("copy_read_only"):
        out["hbm"]["frac_of_measured_read_peak"] = round(gbs / pk["copy_read_only"], 4)
    if pk.get("mfma_bf16_loop"):
        out["mfma"]["frac_of_measured_mfma_peak"] = round(tfs / pk["mfma_bf16_loop"], 4)
    return out


class Workload:
    """One configuration: a learner, its synthetic rollout resident in HBM, and the step that is timed."""

    def __init__(self, idx: int, phase: str, num_envs=None, max_chunk=0, keep_host_samples=0):
        import torch
        from paper_2509_16434_amd import configs, learner, synth
        self.torch = torch
        self.cfg = cfg = configs.get_config(idx, num_envs=num_envs)
        self.net, self.N, self.T = cfg["net"], cfg["num_envs"], cfg["horizon"]
        self.hp = dict(cfg["hp"], seed=cfg["seed"])
        self.distill = cfg["kind"] == "distill"
        self.act = phase == "act"
        self.S = self.N * self.T
        self.stream = torch.cuda.Stream()
        self.lrn = learner.Learner(self.net, self.N, self.T, cfg["obs_dtype"], max_chunk=max_chunk, stream=self.stream)
        self.lrn.set_params(synth.init_params(self.net, cfg["seed"]))
        gen = torch.Generator(device="cuda")
        gen.manual_seed(cfg["seed"])
        self.steps_dev, self.host_steps = [], []
        for t in range(self.T):
            d = synth.rollout_step_torch(cfg, gen)
            have = sum(len(h["done"]) for h in self.host_steps)
            if have < keep_host_samples:   # the first rows of the first steps: the oracle's bounded sample
                m = min(self.N, keep_host_samples - have)
                self.host_steps.append({k: v[:m].float().cpu().numpy() if v.dtype != torch.uint8 else v[:m].cpu().numpy() for k, v in d.items()})
            self.steps_dev.append(d)
        self.last_value = torch.randn(self.N, generator=gen, device="cuda")
        self.noise = [torch.randn(self.N, self.net["act_dim"], generator=gen, device="cuda") for _ in range(self.T)] if self.act else None
        torch.cuda.synchronize()

    def writes(self):
        lrn = self.lrn
        for t, d in enumerate(self.steps_dev):
            if self.distill:
                lrn.buffer_write(t, d["obs"], d["proprio"], d["action"])
            else:
                lrn.buffer_write(t, d["obs"], d["proprio"], d["action"], d["logp_old"], d["value"], d["reward"], d["done"])

    def one_step(self):
        lrn, hp = self.lrn, self.hp
        if self.act:
            for t, d in enumerate(self.steps_dev):
                lrn.act(t, d["obs"], d["proprio"], self.noise[t])
                lrn.buffer_write_outcome(t, d["reward"], d["done"])
            return
        self.writes()
        if self.distill:
            lrn.distill_update(hp, want_stats=False)
        else:
            lrn.gae(self.last_value, hp["gamma"], hp["lam"])
            lrn.update(hp, want_stats=False)

    def sync(self):
        self.stream.synchronize()
        self.torch.cuda.synchronize()

    def timed(self, fn, steps, warmup):
        for _ in range(warmup):
            fn()
        self.sync()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        self.sync()
        return (time.perf_counter() - t0) / steps

    def profiled(self, steps):
        """{class: launches, ms, flops, bytes} over `steps` instrumented steps (HIP events on the library's stream)."""
        self.lrn.profile(True)
        for _ in range(steps):
            self.one_step()
        rep = self.lrn.profile_report()
        self.lrn.profile(False)
        return rep

    def close(self):
        self.lrn.close()
        self.steps_dev = self.noise = self.last_value = None
        self.torch.cuda.empty_cache()


def phases_of(rep: dict, steps: int, w: Workload, t_writes: float) -> dict:
    out = {}
    for k in HBM_SIDE_CLASSES:
        if k in rep and rep[k]["ms"] > 0:
            q = rep[k]
            gbs = q["bytes"] / (q["ms"] * 1e-3) / 1e9
            out[k] = dict(gbs=round(gbs, 1), frac_of_hbm_peak=round(gbs / PEAK_HBM_GBS, 5), avg_launch_us=round(q["ms"] / q["launches"] * 1e3, 2),
                          launches_per_step=q["launches"] / steps, algorithmic_bytes_per_launch=round(q["bytes"] / q["launches"], 1))
    if "buffer_write" in rep:
        q = rep["buffer_write"]
        out["buffer_write"]["T_writes_wall_ms"] = round(t_writes * 1e3, 4)   # T x ppo_buffer_write on their own, wall clock
        out["buffer_write"]["T_writes_wall_gbs"] = round(q["bytes"] / steps / t_writes / 1e9, 1)
    return out


def table(rep, steps, ms_per_step, file=sys.stderr):
    tot_ms = sum(r["ms"] for r in rep.values())
    print(f"{'class':<22}{'launches':>9}{'ms/step':>10}{'share':>8}{'TFLOP/s':>10}{'GB/s':>10}", file=file)
    for k in sorted(rep, key=lambda k: -rep[k]["ms"]):
        q = rep[k]
        sec = q["ms"] * 1e-3
        print(f"{k:<22}{q['launches'] // steps:>9}{q['ms'] / steps:>10.4f}{q['ms'] / tot_ms:>8.3f}"
              f"{q['flops'] / sec / 1e12 if sec else 0:>10.2f}{q['bytes'] / sec / 1e9 if sec else 0:>10.1f}", file=file)
    print(f"kernel time {tot_ms / steps:.3f} ms/step vs wall {ms_per_step:.3f} ms/step", file=file)


def cpu_baseline(w: Workload, n_cpu: int) -> dict:
    """The oracle as it stands on a bounded sample of the workload: forward + loss + backward of n_sub samples on
    all host cores (and of n_sub / cores samples on one thread), GAE and the permutations at full size,
    extrapolated linearly in samples to the whole update."""
    from oracle import ppo_oracle as orc
    from paper_2509_16434_amd import synth
    net, hp, S, T, N = w.net, w.hp, w.S, w.T, w.N
    sub = {k: np.concatenate([h[k] for h in w.host_steps]) for k in w.host_steps[0]}
    n_sub = min(n_cpu, len(sub["done"]))
    p = synth.init_params(net, w.cfg["seed"])

    def net_pass(n):
        t1 = time.perf_counter()
        if w.act:
            orc.act(net, p, sub["obs"][:n], sub["proprio"][:n], np.zeros((n, net["act_dim"])))
        elif w.distill:
            orc.distill_loss_grad(net, p, sub["obs"][:n], sub["proprio"][:n], sub["action"][:n])
        else:
            orc.ppo_loss_grad(net, p, sub["obs"][:n], sub["proprio"][:n], sub["action"][:n], sub["logp_old"][:n], sub["value"][:n],
                              np.zeros(n), np.zeros(n), clip_eps=hp["clip_eps"], vclip_eps=hp["vclip_eps"],
                              vf_coef=hp["vf_coef"], ent_coef=hp["ent_coef"])
        return time.perf_counter() - t1

    def small_parts():
        t2 = time.perf_counter()
        if not w.distill and not w.act:
            z = np.zeros((T, N))
            orc.gae(z, np.zeros((T, N), np.uint8), z, np.zeros(N), hp["gamma"], hp["lam"])
        for e in range(0 if w.act else hp["epochs"]):
            orc.permutation(hp["seed"], 0, e, S)
        return time.perf_counter() - t2

    cores = orc.num_threads()
    passes = 1 if w.act else hp["epochs"]
    t_mb = net_pass(n_sub)
    t_small = small_parts()
    full = t_mb / n_sub * S * passes + t_small
    out = dict(value=round(S / full, 3), unit="env-steps/s", cores=cores, kind="oracle",
               sample=f"{'policy step' if w.act else 'forward+loss+backward'} of {n_sub} of the {S} samples of {w.cfg['name']} timed ({t_mb:.1f} s), "
                      f"extrapolated linearly to {passes} pass(es) over all samples; GAE and permutations timed at full size ({t_small:.2f} s)")
    n1 = max(4, n_sub // max(cores, 1))
    orc.set_num_threads(1)
    try:
        t1 = net_pass(n1)
    finally:
        orc.set_num_threads(cores)
    full1 = t1 / n1 * S * passes + t_small
    out["single_thread"] = dict(value=round(S / full1, 3), unit="env-steps/s", cores=1,
                                sample=f"the same on one thread, {n1} samples timed ({t1:.1f} s)")
    return out


def run_peaks(args):
    """What plain kernels of the library reach on this GPU: a streaming copy, its read-only and store-only halves,
    and a register-resident bf16 MFMA loop.  One JSON line; profiles/peaks.md is made from it."""
    import torch
    from paper_2509_16434_amd import learner
    torch.cuda.set_device(0)
    out = {"metric": "plain-kernel peaks", "n_gpus": 1, "published": {"hbm_gbs": PEAK_HBM_GBS, "mfma_bf16_tflops": PEAK_MFMA_BF16_TF}}
    # 2 GiB per stream: far beyond the 256 MB last-level cache, so these are HBM rates; 128 MiB per stream stays inside it
    for kind in ("copy", "copy_read_only", "copy_write_only", "copy_nt"):
        out[kind] = round(learner.diag_peak(kind, nbytes=2 << 30, iters=20), 1)
        out[kind + "_128MiB"] = round(learner.diag_peak(kind, nbytes=128 << 20, iters=100), 1)
    out["mfma_bf16_loop"] = round(learner.diag_peak("mfma_bf16_loop", iters=20), 1)
    # one 16x16x32 MFMA (16 cycles) + K independent vector instructions per group: do they run side by side on a SIMD?
    for k in (0, 1, 2, 3, 4, 6, 8):
        out[f"mfma16_valu_k{k}"] = round(learner.diag_peak("mfma_valu_loop", nbytes=k, iters=20), 1)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=4, help="index into the benchmark config list (default 4: c4_large, the largest single-GPU workload)")
    ap.add_argument("--num-envs", type=int, default=None, help="override the config's env count (debugging only)")
    ap.add_argument("--max-chunk", type=int, default=0, help="samples per forward/backward pass inside a minibatch (0: the library's default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-per-config", action="store_true", help="only the headline workload")
    ap.add_argument("--phase", choices=["learn", "act", "peaks"], default="learn", help="learn: the learner path (default); act: the policy step; peaks: plain-kernel peaks")
    ap.add_argument("--profile-table", action="store_true", help="also print the per-kernel-class table to stderr")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); run with --gpus 1. "
              "Multi-GPU figures are not produced.", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2509_16434_amd import configs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback.", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.phase == "peaks":
        return run_peaks(args)
    if args.phase == "act" and configs.get_config(args.config)["kind"] == "distill":
        print("bench.py: --phase act needs an actor-critic workload", file=sys.stderr)
        sys.exit(2)

    fl = configs.flops_per_sample(configs.get_config(args.config)["net"])
    n_cpu = int(max(8, 4.0e11 / fl["fwd_bwd"]))  # ~4e11 FLOPs of oracle work, about 10-30 s of CPU time
    w = Workload(args.config, args.phase, args.num_envs, args.max_chunk, keep_host_samples=0 if args.no_cpu_baseline else n_cpu)
    cfg, net, N, T, S, hp = w.cfg, w.net, w.N, w.T, w.S, w.hp
    sec = w.timed(w.one_step, args.steps, args.warmup)
    ms_per_step, value = sec * 1e3, S / sec
    rep = w.profiled(args.steps)
    roofline = roofline_of(rep, cfg["name"], args.steps, use_traffic=args.num_envs is None and not w.act)
    t_writes = w.timed(w.writes, max(args.steps, 3), 1) if not w.act else 0.0
    phases = phases_of(rep, args.steps, w, t_writes) if not w.act else {}
    if args.profile_table:
        table(rep, args.steps, ms_per_step)
    step_flops = fl["fwd"] * S if w.act else fl["fwd_bwd"] * S * hp["epochs"]
    cpu = None if args.no_cpu_baseline else cpu_baseline(w, n_cpu)
    w.close()

    per_config = []
    if not args.no_per_config and args.phase == "learn" and args.num_envs is None:
        for ci in range(len(configs.CONFIGS)):
            if ci == args.config:
                continue
            k = PER_CONFIG_STEPS.get(ci, 3)
            x = Workload(ci, "learn")
            s = x.timed(x.one_step, k, 1)
            r = x.profiled(k)
            rf = roofline_of(r, x.cfg["name"], k, use_traffic=True)
            f2 = configs.flops_per_sample(x.net)["fwd_bwd"] * x.S * x.hp["epochs"]
            per_config.append(dict(workload=x.cfg["name"], num_envs=x.N, horizon=x.T, steps=k, ms_per_step=round(s * 1e3, 4),
                                   value=round(x.S / s, 1), unit="env-steps/s", achieved_tflops=round(f2 / s / 1e12, 3),
                                   mfma_frac_of_peak=round(f2 / s / 1e12 / PEAK_MFMA_BF16_TF, 5),
                                   dominant_kernel=rf["kernel"], bound=rf["bound"], frac=rf["frac"], hbm_frac=rf["hbm"]["frac"],
                                   mfma_frac=rf["mfma"]["frac"], avg_launch_us=rf["avg_launch_us"], traffic=rf["traffic"],
                                   algorithmic_bytes_per_launch=rf["algorithmic_bytes_per_launch"],
                                   phases={p: v["gbs"] for p, v in phases_of(r, k, x, 1.0).items() if p in ("buffer_write", "gae", "adam")}))
            if args.profile_table:
                print(f"--- {x.cfg['name']}", file=sys.stderr)
                table(r, k, s * 1e3)
            x.close()

    out = {
        "metric": "policy env-steps/sec (act + buffer append)" if w.act else
                  "learner env-steps/sec (GAE + PPO epochs)" if not w.distill else "learner env-steps/sec (distillation update)",
        "value": round(value, 1), "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg["name"], "num_envs": N, "horizon": T, "obs": f"{net['n_views']}x{net['in_c']}x{net['in_h']}x{net['in_w']} {cfg['obs_dtype']}",
                   "epochs": hp["epochs"], "minibatches": hp["minibatches"], "params": configs.param_count(net)},
        "achieved_tflops": round(step_flops / sec / 1e12, 3),
        "mfma_frac_of_peak": round(step_flops / sec / 1e12 / PEAK_MFMA_BF16_TF, 5),
        "roofline": roofline, "cpu_baseline": cpu, "phases": phases, "per_config": per_config,
        "peaks_measured": measured_peaks() or None,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
