"""GPU parity tests: every entry point of libppo_learner.so against the CPU oracle on the same
seeded inputs.  Tolerances: GAE/returns 1e-5 (fp32); losses, gradients and updated parameters
2e-2 (bf16 MFMA with fp32 accumulation; per-tensor relative L2 for tensors); permutations and
the stored bf16 images bit-exact.

Network outputs and loss statistics are held to 2e-2 against the oracle's exact fp64 mode.
Gradients and updated parameters are held to 2e-2 against the oracle's bf16-operand mode (same
formulas, operands rounded to bf16 where the kernels store bf16, fp64 accumulation): the ReLU
masks and the active branch of the clipped losses are discrete decisions and both sides must take
them in the same precision.  Against the exact mode the gradients of these synthetic rollouts
(pure-noise returns, so the batch gradient is a sqrt(B)-cancelled sum) differ by a few percent
for ANY bf16-operand implementation; that distance is checked against a loose bound only."""
import numpy as np
import pytest

from oracle import ppo_oracle as orc
from paper_2509_16434_amd import configs, synth

from helpers import TOL_BF16, TOL_GAE, fill_learner, flat_rollout, per_tensor_errors, per_tensor_param_errors, rel_l2

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def L():
    from paper_2509_16434_amd import learner
    return learner


def _torch():
    import torch
    return torch


def _setup(L, cfg, max_chunk=0, seed=None):
    ro = synth.rollout(cfg, seed)
    lrn = L.Learner(cfg["net"], cfg["num_envs"], cfg["horizon"], cfg["obs_dtype"], max_chunk=max_chunk)
    params = synth.init_params(cfg["net"], cfg["seed"])
    lrn.set_params(params)
    fill_learner(lrn, cfg, ro, distill=(cfg["kind"] == "distill"))
    return lrn, ro, params


# ------------------------------------------------------------------ MFMA tile kernel
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (200, 24, 72), (300, 64, 288), (129, 130, 8), (64, 512, 1056), (1, 1, 8),
                                   (300, 40, 1032), (129, 20, 2048), (32773, 48, 1024),
                                   (32768 + 37, 250, 1096)])  # the last: 256 x 128 tiles, eight compute waves
def test_mfma_gemm_tiles(L, M, N, K):
    rng = np.random.default_rng(M * 7 + N)
    a = synth.narrow_bf16(rng.standard_normal((M, K)).astype(np.float32))
    b = synth.narrow_bf16(rng.standard_normal((N, K)).astype(np.float32))
    c = L.diag_gemm(a, b)
    want = a.astype(np.float64) @ b.astype(np.float64).T
    assert np.abs(c - want).max() <= 1e-4 * max(1.0, np.abs(want).max())


def test_peak_diagnostics_run(L):
    """The plain kernels behind `bench.py --phase peaks`: each kind returns a positive rate; more vector instructions per
    MFMA never make the MFMA loop faster."""
    assert L.diag_peak("copy", nbytes=64 << 20, iters=2) > 100.0
    assert L.diag_peak("mfma_bf16_loop", iters=2) > 100.0
    r0 = L.diag_peak("mfma_valu_loop", nbytes=0, iters=3)
    r8 = L.diag_peak("mfma_valu_loop", nbytes=8, iters=3)
    assert r0 > 100.0 and 0.0 < r8 <= r0 * 1.02


# ------------------------------------------------------------------ buffer
@pytest.mark.parametrize("ci", [0, 1, 3])
def test_buffer_write_read_back(L, ci):
    torch = _torch()
    cfg = configs.get_config(ci, num_envs=24, horizon=2)
    lrn, ro, _ = _setup(L, cfg)
    for t in range(cfg["horizon"]):
        got = lrn.buffer_read_obs(t).to(torch.float32).cpu().numpy()
        want = torch.from_numpy(ro["obs"][t]).to(torch.bfloat16).to(torch.float32).numpy()
        np.testing.assert_array_equal(got, want)
    net = cfg["net"]
    assert lrn.buffer_image_bytes() == orc.buffer_image_bytes(24, 2, net["n_views"], net["in_c"], net["in_h"], net["in_w"], 2)


def test_buffer_write_odd_image_size(L):
    torch = _torch()
    cfg = configs.get_config(0, num_envs=5, horizon=2)
    cfg["net"].update(in_h=9, in_w=11)
    lrn, ro, _ = _setup(L, cfg)
    got = lrn.buffer_read_obs(1).to(torch.float32).cpu().numpy()
    want = torch.from_numpy(ro["obs"][1]).to(torch.bfloat16).to(torch.float32).numpy()
    np.testing.assert_array_equal(got, want)


def test_buffer_write_by_environment_ranges(L):
    """Slabs filled by several producers (ragged, out-of-order environment ranges) hold exactly what one full
    write leaves: stored images bit for bit, and a whole update from them bit-identical parameters."""
    torch = _torch()
    cfg = configs.get_config(0, num_envs=50, horizon=4)
    cfg["net"].update(in_h=9, in_w=11)      # 99-element images: slices start at odd element offsets
    hp = dict(cfg["hp"], epochs=1, minibatches=2, seed=5)
    full, ro, params = _setup(L, cfg)
    part = L.Learner(cfg["net"], 50, 4, cfg["obs_dtype"])
    part.set_params(params)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bounds = [(37, 50), (0, 1), (8, 37), (1, 8)]
    lv = dev(ro["last_value"])
    for t in range(4):
        for i, (a, b) in enumerate(bounds):
            if i == len(bounds) - 1:    # one range still missing: the rollout is not complete
                with pytest.raises(L.LearnerError) as e:
                    part.gae(lv, hp["gamma"], hp["lam"])
                assert e.value.code == L.PPO_ESTATE
            part.buffer_write_range(t, a, dev(ro["obs"][t][a:b]), *[dev(ro[k][t][a:b]) for k in
                                    ("proprio", "action", "logp_old", "value", "reward", "done")])
    for t in range(4):
        assert torch.equal(part.buffer_read_obs(t), full.buffer_read_obs(t))
    for x in (full, part):
        x.gae(lv, hp["gamma"], hp["lam"])
        x.update(hp)
    np.testing.assert_array_equal(part.get_params(), full.get_params())
    with pytest.raises(L.LearnerError) as e:
        part.buffer_write_range(0, 40, dev(ro["obs"][0][:11]), *[dev(ro[k][0][:11]) for k in
                                ("proprio", "action", "logp_old", "value", "reward", "done")])
    assert e.value.code == L.PPO_EINVAL
    # a range that arrives when the whole rollout is complete begins the NEXT rollout: no step counts as written
    # (the slabs still hold the first rollout) until its own ranges cover all environments again
    ro2 = synth.rollout(cfg, seed=cfg["seed"] + 1)
    fields = ("proprio", "action", "logp_old", "value", "reward", "done")
    part.buffer_write_range(2, 0, dev(ro2["obs"][2][:5]), *[dev(ro2[k][2][:5]) for k in fields])
    with pytest.raises(L.LearnerError) as e:
        part.gae(lv, hp["gamma"], hp["lam"])
    assert e.value.code == L.PPO_ESTATE
    part.buffer_write_range(2, 5, dev(ro2["obs"][2][5:]), *[dev(ro2[k][2][5:]) for k in fields])   # step 2 complete, 0, 1, 3 are not
    for t in (3, 1):
        for a, b in ((25, 50), (0, 25)):
            part.buffer_write_range(t, a, dev(ro2["obs"][t][a:b]), *[dev(ro2[k][t][a:b]) for k in fields])
    with pytest.raises(L.LearnerError) as e:    # step 0 still holds only the first rollout's record
        part.gae(lv, hp["gamma"], hp["lam"])
    assert e.value.code == L.PPO_ESTATE
    with pytest.raises(L.LearnerError) as e:
        part.buffer_read_obs(0)
    assert e.value.code == L.PPO_ESTATE
    # within a rollout (step 0 is still missing), a partial write into a complete step makes that step incomplete again
    part.buffer_write_range(3, 10, dev(ro2["obs"][3][10:20]), *[dev(ro2[k][3][10:20]) for k in fields])
    with pytest.raises(L.LearnerError) as e:
        part.buffer_read_obs(3)
    assert e.value.code == L.PPO_ESTATE
    for a, b in ((0, 10), (20, 50)):
        part.buffer_write_range(3, a, dev(ro2["obs"][3][a:b]), *[dev(ro2[k][3][a:b]) for k in fields])
    assert torch.equal(part.buffer_read_obs(3), dev(ro2["obs"][3]).to(torch.bfloat16))
    part.buffer_write_range(0, 0, dev(ro2["obs"][0]), *[dev(ro2[k][0]) for k in fields])
    fill_learner(full, cfg, ro2)
    lv2 = dev(ro2["last_value"])
    for x in (full, part):
        x.gae(lv2, hp["gamma"], hp["lam"])
        x.update(hp)
    np.testing.assert_array_equal(part.get_params(), full.get_params())


# ------------------------------------------------------------------ GAE
@pytest.mark.parametrize("N,T", [(64, 16), (1000, 16), (16384, 32), (1, 1), (3, 7)])
def test_gae_matches_oracle(L, N, T):
    torch = _torch()
    cfg = configs.get_config(0, num_envs=N, horizon=T)
    cfg["net"].update(in_h=8, in_w=8)
    rng = np.random.default_rng(N + T)
    lrn = L.Learner(cfg["net"], N, T, "fp32")
    r = rng.standard_normal((T, N)).astype(np.float32)
    v = rng.standard_normal((T, N)).astype(np.float32)
    d = (rng.random((T, N)) < 0.05).astype(np.uint8)
    lv = rng.standard_normal(N).astype(np.float32)
    net = cfg["net"]
    z = lambda *s: torch.zeros(*s, device="cuda")
    obs = z(N, 1, 1, 8, 8)
    for t in range(T):
        lrn.buffer_write(t, obs, z(N, net["proprio_dim"]), z(N, net["act_dim"]), z(N), torch.from_numpy(v[t]).cuda(),
                         torch.from_numpy(r[t]).cuda(), torch.from_numpy(d[t]).cuda())
    lrn.gae(torch.from_numpy(lv).cuda(), 0.99, 0.95)
    adv, ret = lrn.get_adv_ret()
    oadv, oret = orc.gae(r, d, v, lv, 0.99, 0.95)
    for got, want in ((adv, oadv), (ret, oret)):
        got = got.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - want) <= TOL_GAE * np.maximum(1.0, np.abs(want)))
    # returns are one fp32 add on top of the advantage
    np.testing.assert_array_equal(ret.cpu().numpy(), adv.cpu().numpy() + v)


# ------------------------------------------------------------------ permutation
@pytest.mark.parametrize("S", [1, 37, 1024, 16384, 65536, 524288])
def test_permutation_bit_exact(L, S):
    cfg = configs.get_config(0, num_envs=S, horizon=1)
    cfg["net"].update(in_h=2, in_w=2)
    lrn = L.Learner(cfg["net"], S, 1, "fp32")
    for (seed, upd, ep) in [(0, 0, 0), (1234, 5, 3)]:
        got = lrn.permutation(seed, upd, ep)
        np.testing.assert_array_equal(got, orc.permutation(seed, upd, ep, S))


# ------------------------------------------------------------------ forward
FWD_CASES = [(0, 64, 16), (1, 40, 4), (2, 12, 4), (3, 8, 4), (5, 6, 2)]


@pytest.mark.parametrize("ci,N,T", FWD_CASES)
def test_forward_matches_oracle(L, ci, N, T):
    cfg = configs.get_config(ci, num_envs=N, horizon=T)
    lrn, ro, params = _setup(L, cfg)
    fr = flat_rollout(ro)
    mu, v = lrn.forward()
    omu, ov = orc.forward(cfg["net"], params, fr["obs"], fr["proprio"])
    assert rel_l2(mu.cpu().numpy(), omu) <= TOL_BF16
    if v is not None:
        assert rel_l2(v.cpu().numpy(), ov) <= TOL_BF16
    with orc.quant(1):
        qmu, qv = orc.forward(cfg["net"], params, fr["obs"], fr["proprio"])
    assert rel_l2(mu.cpu().numpy(), qmu) <= 5e-3
    if v is not None:
        assert rel_l2(v.cpu().numpy(), qv) <= 5e-3


# ------------------------------------------------------------------ policy step of the collection loop
ACT_CASES = [(0, 64, 3), (1, 200, 2), (1, 1024, 2), (2, 24, 2)]  # (1, 1024, .) is the benchmark's shape


@pytest.mark.parametrize("ci,N,T", ACT_CASES)
def test_act_matches_oracle_and_fills_the_buffer(L, ci, N, T):
    torch = _torch()
    cfg = configs.get_config(ci, num_envs=N, horizon=T)
    net, A = cfg["net"], cfg["net"]["act_dim"]
    ro = synth.rollout(cfg)
    params = synth.init_params(net, cfg["seed"])
    a0, a1, _ = synth.param_slices(net)["logstd"]
    rng = np.random.default_rng(99)
    params[a0:a1] = rng.uniform(-1.0, 0.5, A).astype(np.float32)
    sigma = np.exp(params[a0:a1].astype(np.float64))
    lrn = L.Learner(net, N, T, cfg["obs_dtype"])
    lrn.set_params(params)
    odt = torch.float32 if cfg["obs_dtype"] == "fp32" else torch.bfloat16
    noise = rng.standard_normal((T, N, A)).astype(np.float32)
    acted = []
    for t in range(T):
        obs = torch.from_numpy(ro["obs"][t]).cuda().to(odt).contiguous()
        pr = torch.from_numpy(ro["proprio"][t]).cuda().contiguous()
        a, lp, v = lrn.act(t, obs, pr, torch.from_numpy(noise[t]).cuda())
        lrn.synchronize()
        a, lp, v = a.cpu().numpy(), lp.cpu().numpy(), v.cpu().numpy()
        acted.append((a, lp, v))
        oa, olp, ov = orc.act(net, params, ro["obs"][t], ro["proprio"][t], noise[t])
        omu = oa - sigma * noise[t]
        # the sampled offset is common to both sides: the error is measured against the mean's norm
        assert np.linalg.norm(a - oa) / np.linalg.norm(omu) <= TOL_BF16
        assert rel_l2(v, ov) <= TOL_BF16
        assert np.max(np.abs(lp - olp)) <= 1e-3
        with orc.quant(1):
            qa, _, qv = orc.act(net, params, ro["obs"][t], ro["proprio"][t], noise[t])
        assert np.linalg.norm(a - qa) / np.linalg.norm(omu) <= 5e-3 and rel_l2(v, qv) <= 5e-3
    # gae is refused until every step has its outcome
    lv = torch.from_numpy(ro["last_value"]).cuda()
    with pytest.raises(L.LearnerError) as e:
        lrn.gae(lv, 0.99, 0.95)
    assert e.value.code == L.PPO_ESTATE
    for t in range(T):
        lrn.buffer_write_outcome(t, torch.from_numpy(ro["reward"][t]).cuda(), torch.from_numpy(ro["done"][t]).cuda())
    lrn.gae(lv, cfg["hp"]["gamma"], cfg["hp"]["lam"])
    # the slab holds what act returned: GAE from the returned values equals the oracle's
    vals = np.stack([x[2] for x in acted])
    adv, ret = lrn.get_adv_ret()
    oadv, oret = orc.gae(ro["reward"], ro["done"], vals, ro["last_value"], cfg["hp"]["gamma"], cfg["hp"]["lam"])
    assert np.max(np.abs(adv.cpu().numpy() - oadv) / np.maximum(1, np.abs(oadv))) <= TOL_GAE
    # and the stored actions and log-probs give ratio 1 on the first optimiser step
    if (N * T) % 2 == 0:
        st = lrn.update(dict(cfg["hp"], epochs=1, minibatches=2))
        assert abs(st[0]["approx_kl"]) <= 1e-6 and st[0]["clip_frac"] == 0.0
        B = N * T // 2
        perm = orc.permutation(cfg["hp"].get("seed", 0), 0, 0, N * T)[:B]
        assert abs(st[0]["pi_loss"] + oadv.reshape(-1)[perm].mean()) <= 1e-4 * max(1.0, np.abs(oadv).max())


def test_act_in_chunks_equals_one_pass(L):
    """More environments than the chunk of the forward workspaces: the chunk loop of ppo_act gives the same
    actions, log-probs and values, bit for bit, as one pass."""
    torch = _torch()
    cfg = configs.get_config(1, num_envs=150, horizon=1)
    ro = synth.rollout(cfg)
    params = synth.init_params(cfg["net"], cfg["seed"])
    obs = torch.from_numpy(ro["obs"][0]).cuda().to(torch.bfloat16).contiguous()
    pr = torch.from_numpy(ro["proprio"][0]).cuda().contiguous()
    noise = torch.randn(150, cfg["net"]["act_dim"], device="cuda", generator=torch.Generator(device="cuda").manual_seed(3))
    outs = []
    for chunk in (0, 64):
        lrn = L.Learner(cfg["net"], 150, 1, cfg["obs_dtype"], max_chunk=chunk)
        lrn.set_params(params)
        a, lp, v = lrn.act(0, obs, pr, noise)
        lrn.synchronize()
        outs.append((a.cpu().numpy(), lp.cpu().numpy(), v.cpu().numpy()))
    for x, y in zip(*outs):
        np.testing.assert_array_equal(x, y)


def test_act_call_order_errors(L):
    torch = _torch()
    cfg = configs.get_config(0, num_envs=8, horizon=2)
    lrn = L.Learner(cfg["net"], 8, 2, "fp32")
    z = torch.zeros(8, device="cuda")
    with pytest.raises(L.LearnerError) as e:
        lrn.buffer_write_outcome(0, z, z.to(torch.uint8))
    assert e.value.code == L.PPO_ESTATE
    scfg = _stereo_cfg(8, 2)
    stu = L.Learner(scfg["net"], 8, 2, scfg["obs_dtype"])
    sn = scfg["net"]
    with pytest.raises(L.LearnerError) as e:
        stu.act(0, torch.zeros(8, sn["n_views"], sn["in_c"], sn["in_h"], sn["in_w"], device="cuda", dtype=torch.bfloat16),
                torch.zeros(8, sn["proprio_dim"], device="cuda"), torch.zeros(8, sn["act_dim"], device="cuda"))
    assert e.value.code == L.PPO_ESTATE


# ------------------------------------------------------------------ one minibatch: loss and gradients
def _oracle_inputs(cfg, ro, lrn):
    fr = flat_rollout(ro)
    adv, ret = orc.gae(ro["reward"], ro["done"], ro["value"], ro["last_value"], cfg["hp"]["gamma"], cfg["hp"]["lam"])
    return fr, adv.reshape(-1), ret.reshape(-1)


# minibatches of >= 160 samples: below that the ulp-level ReLU-mask differences between two bf16-operand
# implementations show up in the noise-label gradient (~1/sqrt(B): 2.5 % at B = 48, 0.5 % at B = 192)
GRAD_CASES = [(0, 64, 16, 0), (0, 64, 16, 100), (1, 40, 4, 0), (2, 64, 4, 0), (2, 64, 4, 100), (5, 48, 4, 0)]


@pytest.mark.parametrize("ci,N,T,chunk", GRAD_CASES)
def test_ppo_single_minibatch_gradients(L, ci, N, T, chunk):
    _check_single_minibatch(L, configs.get_config(ci, num_envs=N, horizon=T), chunk)


# Shapes that exercise the ragged paths of the LDS-image convolution kernels: odd heights and widths
# (last quad row / column without a partner, right zero-pad pixel in use), bands that do not divide the
# image, an image height whose first-layer output is odd.
# (50, 96) and (36, 80) have a first-layer output width that is a multiple of 8: the register-fused
# first-layer weight gradient takes them (odd output height, bands that do not divide the image).
ODD_SHAPES = [(52, 76), (50, 72), (44, 88), (50, 96), (36, 80),
              # small and tall images, an odd height, several bands per image, rows of 13 to 15 sixteen-byte pieces
              (24, 40), (70, 56), (33, 64), (16, 16), (90, 120), (28, 104),
              # very wide rows: one quad row per band in the register-fused kernel, whose loader waves then share the
              # 1 KiB parts of every gradient row (20 parts; 17 parts with a last part of 512 bytes)
              (24, 640), (20, 528)]


@pytest.mark.parametrize("h,w", ODD_SHAPES)
def test_ppo_gradients_odd_image_shapes(L, h, w):
    cfg = configs.get_config(1, num_envs=48, horizon=4)
    cfg["net"].update(in_h=h, in_w=w)
    # (the distance to exact arithmetic is a property of bf16 operands on the sampled batch, not of the
    # kernels: the same gradient is within 2e-2 of the oracle's bf16-operand mode; it is only bounded loosely)
    _check_single_minibatch(L, cfg, 0, loose_bound=0.3)


def _check_single_minibatch(L, cfg, chunk, loose_bound=0.15):
    torch = _torch()
    lrn, ro, params = _setup(L, cfg, max_chunk=chunk)
    hp = dict(cfg["hp"], epochs=1, minibatches=1, seed=3)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    st = lrn.update(hp)[0]
    g = lrn.get_grads()
    fr, adv, ret = _oracle_inputs(cfg, ro, lrn)
    args = (cfg["net"], params, fr["obs"], fr["proprio"], fr["action"], fr["logp_old"], fr["value"], adv, ret)
    kw = dict(clip_eps=hp["clip_eps"], vclip_eps=hp["vclip_eps"], vf_coef=hp["vf_coef"], ent_coef=hp["ent_coef"])
    with orc.quant(1):
        qst, qg = orc.ppo_loss_grad(*args, **kw)      # bf16 operands, fp64 accumulation
    ost, og = orc.ppo_loss_grad(*args, **kw) if chunk == 0 else (qst, qg)   # exact fp64 (once per net)
    for ref in (ost, qst):
        for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("entropy", "entropy"), ("approx_kl", "approx_kl"),
                            ("clip_frac", "clip_frac"), ("total_loss", "total")):
            assert abs(st[k_gpu] - ref[k_or]) <= TOL_BF16 * max(abs(ref[k_or]), 1e-3), (k_gpu, st[k_gpu], ref[k_or])
    assert abs(st["grad_norm"] - qst["grad_norm"]) <= TOL_BF16 * qst["grad_norm"]
    assert st["nonfinite"] == 0
    errs = per_tensor_errors(cfg["net"], g, qg)
    assert max(errs.values()) <= TOL_BF16, errs
    # distance to the exact-arithmetic gradient: bf16 operand rounding on a noise-dominated batch gradient
    loose = per_tensor_errors(cfg["net"], g, og)
    assert max(loose.values()) <= loose_bound, loose


def test_full_size_bench_minibatch_matches_oracle(L):
    """The benchmark's default workload at its full size and in its launch configuration (1024 envs x 16
    steps, minibatches of 4096 samples, one chunk each).  With lr = 0 the parameters never move, so the
    gradient left after the update is the initial-parameter gradient of the LAST minibatch of the epoch,
    whose samples the oracle takes from the (bit-exact) permutation; its statistics are step 3's."""
    torch = _torch()
    cfg = configs.get_config(1)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], epochs=1, minibatches=4, seed=11, lr=0.0)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    stats = lrn.update(hp)
    np.testing.assert_array_equal(lrn.get_params(), params)
    g = lrn.get_grads()
    S = cfg["num_envs"] * cfg["horizon"]
    perm = orc.permutation(hp["seed"], 0, 0, S)
    B = S // 4
    sel = perm[3 * B:]
    fr, adv, ret = _oracle_inputs(cfg, ro, lrn)
    with orc.quant(1):
        qst, qg = orc.ppo_loss_grad(cfg["net"], params, fr["obs"][sel], fr["proprio"][sel], fr["action"][sel], fr["logp_old"][sel],
                                    fr["value"][sel], adv[sel], ret[sel], clip_eps=hp["clip_eps"], vclip_eps=hp["vclip_eps"],
                                    vf_coef=hp["vf_coef"], ent_coef=hp["ent_coef"])
    st = stats[3]
    for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("approx_kl", "approx_kl"), ("clip_frac", "clip_frac"), ("total_loss", "total")):
        assert abs(st[k_gpu] - qst[k_or]) <= TOL_BF16 * max(abs(qst[k_or]), 1e-3), (k_gpu, st[k_gpu], qst[k_or])
    assert abs(st["grad_norm"] - qst["grad_norm"]) <= TOL_BF16 * qst["grad_norm"]
    errs = per_tensor_errors(cfg["net"], g, qg)
    assert max(errs.values()) <= TOL_BF16, errs


@pytest.mark.parametrize("ci", [2, 3, 4])
def test_full_size_sampled_outputs(L, ci):
    """The paper-scale workloads (c2: 4096 envs x 16 steps of 120x160 depth, 2.5 GB of buffered images; c3: the
    stereo-RGB student, 15 GB; c4: 16384 envs x 32 steps, 20 GB) at full size and in the default launch
    configuration, on sampled outputs the oracle computes one by one: network outputs of 24 samples spread over
    the buffer, advantages and returns of 16 environments, the stored images of one step bit for bit; then
    properties that hold at any size.  The rollout is drawn on the GPU (seeded) as the benchmark does."""
    torch = _torch()
    cfg = configs.get_config(ci)
    net, N, T = cfg["net"], cfg["num_envs"], cfg["horizon"]
    distill = cfg["kind"] == "distill"
    lrn = L.Learner(net, N, T, cfg["obs_dtype"])
    params = synth.init_params(net, cfg["seed"])
    lrn.set_params(params)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(cfg["seed"])
    rng = np.random.default_rng(5)
    sel = np.sort(rng.choice(N * T, 24, replace=False))
    envs = np.sort(rng.choice(N, 16, replace=False))
    keep = {int(s): None for s in sel}
    scal = {k: np.empty((T, len(envs)), np.float64) for k in ("reward", "value")}
    done = np.empty((T, len(envs)), np.uint8)
    for t in range(T):
        d = synth.rollout_step_torch(cfg, gen)
        if distill:
            lrn.buffer_write(t, d["obs"], d["proprio"], d["action"])
        else:
            lrn.buffer_write(t, d["obs"], d["proprio"], d["action"], d["logp_old"], d["value"], d["reward"], d["done"])
        for s in sel[(sel >= t * N) & (sel < (t + 1) * N)]:
            n = int(s) - t * N
            keep[int(s)] = (d["obs"][n].float().cpu().numpy(), d["proprio"][n].cpu().numpy().astype(np.float64))
        for k in scal:
            scal[k][t] = d[k][envs].cpu().numpy()
        done[t] = d["done"][envs].cpu().numpy()
        if t == T // 2:
            assert torch.equal(lrn.buffer_read_obs(t), d["obs"])
        del d
    if not distill:
        last_value = torch.randn(N, generator=gen, device="cuda")
        lrn.gae(last_value, cfg["hp"]["gamma"], cfg["hp"]["lam"])
        adv, ret = lrn.get_adv_ret()
        oadv, oret = orc.gae(scal["reward"], done, scal["value"], last_value[envs].cpu().numpy().astype(np.float64),
                             cfg["hp"]["gamma"], cfg["hp"]["lam"])
        for got, want in ((adv, oadv), (ret, oret)):
            gsel = got[:, envs].cpu().numpy()
            assert np.max(np.abs(gsel - want) / np.maximum(1, np.abs(want))) <= TOL_GAE
    mu, v = lrn.forward(idx=torch.from_numpy(sel.astype(np.int32)).cuda())
    obs = np.stack([keep[int(s)][0] for s in sel])
    pro = np.stack([keep[int(s)][1] for s in sel])
    omu, ov = orc.forward(net, params, obs, pro)
    with orc.quant(1):
        qmu, qv = orc.forward(net, params, obs, pro)
    assert rel_l2(mu.cpu().numpy(), omu) <= TOL_BF16 and rel_l2(mu.cpu().numpy(), qmu) <= 5e-3
    if not distill:
        assert rel_l2(v.cpu().numpy(), ov) <= TOL_BF16 and rel_l2(v.cpu().numpy(), qv) <= 5e-3
    # properties that hold at any size: with lr = 0 an epoch leaves the parameters untouched, its statistics are
    # finite, and a second pass over the same buffer reproduces statistics and gradient bit for bit (the partial
    # sums of the weight gradients are taken in a fixed order)
    hp = dict(cfg["hp"], epochs=1, lr=0.0, seed=3)
    runs = []
    for _ in range(2):
        lrn.set_opt_state(np.zeros_like(params), np.zeros_like(params), 0, 0)
        st = lrn.distill_update(hp) if distill else lrn.update(hp)
        runs.append((st, lrn.get_grads()))
    np.testing.assert_array_equal(lrn.get_params(), params)
    assert all(x["nonfinite"] == 0 and np.isfinite(x["grad_norm"]) and x["grad_norm"] > 0 for x in runs[0][0])
    assert runs[0][0] == runs[1][0]
    np.testing.assert_array_equal(runs[0][1], runs[1][1])
    lrn.close()


# ------------------------------------------------------------------ Adam, from the library's own gradients
@pytest.mark.parametrize("ci,N,T", [(0, 64, 16), (1, 64, 4)])
def test_adam_steps_replayed_exactly(L, ci, N, T):
    """Two single-minibatch updates; after each, the oracle's Adam applied to the gradient the library
    reports must reproduce the library's parameters and moments to fp32 rounding.  Feeding both sides the
    same gradient removes Adam's sign discontinuity (an element whose gradient is below the bf16 noise
    floor moves by +-lr on the first steps) from the comparison."""
    torch = _torch()
    cfg = configs.get_config(ci, num_envs=N, horizon=T)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], epochs=1, minibatches=1, seed=3)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    p = params.astype(np.float64)
    m, v = np.zeros_like(p), np.zeros_like(p)
    for k in (1, 2):
        lrn.update(hp)
        g = lrn.get_grads().astype(np.float64)
        orc.adam_step(p, m, v, g, k, lr=hp["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["adam_eps"])
        gm, gv, step, upd = lrn.get_opt_state()
        assert step == k and upd == k
        got = lrn.get_params().astype(np.float64)
        # fp32 arithmetic: the step itself (<= lr per element) is reproduced to ~1e-6 of lr-sized quantities
        assert np.abs(got - p).max() <= 1e-6 * max(1.0, np.abs(p).max()) + 2e-3 * hp["lr"]
        # beta2 crosses the ABI as an fp32 number: 1 - 0.999f differs from 1e-3 by 1.3e-5 relative
        assert rel_l2(gm, m) <= 1e-5 and rel_l2(gv, v) <= 5e-5
        p = got.copy()  # continue from the library's fp32 state
        m, v = gm.astype(np.float64), gv.astype(np.float64)


# ------------------------------------------------------------------ optional PPO features
def test_advantage_normalisation_and_grad_clipping(L):
    """One minibatch over the whole rollout with both options on: statistics and gradient against the oracle fed
    with its own normalised advantages; the clipped Adam step replayed exactly from the gradient the library
    reports; a clip threshold above the norm changes nothing, bit for bit."""
    torch = _torch()
    cfg = configs.get_config(0, num_envs=64, horizon=16)
    base = dict(cfg["hp"], epochs=1, minibatches=1, seed=3, norm_adv=1)
    fr = adv = ret = None
    results = {}
    for name, mx in (("off", 0.0), ("loose", 1e6), ("tight", None)):
        lrn, ro, params = _setup(L, cfg)
        lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), base["gamma"], base["lam"])
        if mx is None:
            mx = 0.3 * results["off"][0]["grad_norm"]
        st = lrn.update(dict(base, max_grad_norm=mx))[0]
        results[name] = (st, lrn.get_grads(), lrn.get_params(), lrn.get_opt_state(), mx)
        if fr is None:
            fr, adv, ret = _oracle_inputs(cfg, ro, lrn)
    st, g, p_off, _, _ = results["off"]
    nadv = orc.normalize_adv(adv)
    with orc.quant(1):
        qst, qg = orc.ppo_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"], fr["logp_old"], fr["value"], nadv, ret,
                                    clip_eps=base["clip_eps"], vclip_eps=base["vclip_eps"], vf_coef=base["vf_coef"], ent_coef=base["ent_coef"])
    for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("approx_kl", "approx_kl"), ("clip_frac", "clip_frac"), ("total_loss", "total")):
        assert abs(st[k_gpu] - qst[k_or]) <= TOL_BF16 * max(abs(qst[k_or]), 1e-3), (k_gpu, st[k_gpu], qst[k_or])
    errs = per_tensor_errors(cfg["net"], g, qg)
    assert max(errs.values()) <= TOL_BF16, errs
    # the raw advantages would give a different policy loss: the option is really on
    with orc.quant(1):
        rst, _ = orc.ppo_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"], fr["logp_old"], fr["value"], adv, ret,
                                   clip_eps=base["clip_eps"], vclip_eps=base["vclip_eps"], vf_coef=base["vf_coef"], ent_coef=base["ent_coef"])
    assert abs(rst["pi_loss"] - qst["pi_loss"]) > 10 * TOL_BF16 * max(abs(qst["pi_loss"]), 1e-3)
    # a threshold above the norm: identical to no clipping
    np.testing.assert_array_equal(results["loose"][2], p_off)
    # an active threshold: same gradient and reported (pre-clip) norm, Adam step of the clipped gradient
    stt, gt, pt, (gm, gv, step, _), mx = results["tight"]
    np.testing.assert_array_equal(gt, g)
    assert stt["grad_norm"] == st["grad_norm"] and abs(stt["grad_norm"] - np.linalg.norm(g.astype(np.float64))) <= 1e-5 * stt["grad_norm"]
    clipped, n = orc.clip_grad_norm(g.astype(np.float64), mx)
    assert n > mx
    p = params.astype(np.float64)
    m, v = np.zeros_like(p), np.zeros_like(p)
    orc.adam_step(p, m, v, clipped, 1, lr=base["lr"], beta1=base["beta1"], beta2=base["beta2"], eps=base["adam_eps"])
    assert step == 1
    assert np.abs(pt.astype(np.float64) - p).max() <= 1e-6 * max(1.0, np.abs(p).max()) + 2e-3 * base["lr"]
    assert rel_l2(gm, m) <= 1e-5 and rel_l2(gv, v) <= 5e-5
    assert rel_l2(gm, 0.3 * results["off"][3][0] * (st["grad_norm"] / (st["grad_norm"] + 1e-6))) <= 1e-5   # m scales with the coefficient


# ------------------------------------------------------------------ whole update
def _compare_update(L, cfg, lrn, ro, params, out, stats, lr):
    """Loss statistics of every optimiser step, and the parameters after the whole update.  From the second
    step on the two sides no longer start from identical parameters (Adam's sign discontinuity), and the
    batch gradient of pure-noise returns is very sensitive to that, so the end-of-update parameters are
    compared on the scale max(||theta||, sqrt(n)*steps*lr) of what Adam can have moved."""
    for k, (s, o) in enumerate(zip(stats, out["stats"])):
        for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("total_loss", "total")):
            assert abs(s[k_gpu] - o[k_or]) <= TOL_BF16 * max(abs(o[k_or]), 1e-3), (k_gpu, s[k_gpu], o[k_or])
        # the gradient (unlike the loss) of a later step is sensitive to the sign-noise difference in its
        # starting parameters: tight for the first step, loose afterwards
        assert abs(s["grad_norm"] - o["grad_norm"]) <= (TOL_BF16 if k == 0 else 0.25) * o["grad_norm"], (k, s["grad_norm"], o["grad_norm"])
    assert rel_l2(lrn.get_params(), out["params"]) <= TOL_BF16
    errs = per_tensor_param_errors(cfg["net"], lrn.get_params(), out["params"], len(stats), lr)
    print({k: round(v, 4) for k, v in errs.items() if v > 5e-3})
    assert max(errs.values()) <= 2.5 * TOL_BF16, errs
    d_gpu = lrn.get_params().astype(np.float64) - params
    d_or = out["params"] - params
    cos = float(d_gpu @ d_or / (np.linalg.norm(d_gpu) * np.linalg.norm(d_or)))
    assert cos > 0.95, cos


@pytest.mark.parametrize("ci,N,T,extras", [(0, 64, 16, {}), (1, 256, 4, {}), (0, 64, 16, dict(norm_adv=1, max_grad_norm=0.5))])
def test_ppo_update_matches_oracle(L, ci, N, T, extras):
    torch = _torch()
    cfg = configs.get_config(ci, num_envs=N, horizon=T)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], seed=11, **extras)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    stats = lrn.update(hp)
    fr, adv, ret = _oracle_inputs(cfg, ro, lrn)
    z = np.zeros_like(params, dtype=np.float64)
    with orc.quant(1):
        out = orc.ppo_update(cfg["net"], params, z, z, 0, fr["obs"], fr["proprio"], fr["action"], fr["logp_old"], fr["value"],
                             adv, ret, hp, update_idx=0)
    _compare_update(L, cfg, lrn, ro, params, out, stats, hp["lr"])
    m, v, step, upd = lrn.get_opt_state()
    assert step == out["step"] == hp["epochs"] * hp["minibatches"] and upd == 1


def _rule32(lr, kl, d, lo, hi):
    """The schedule in the kernel's precision."""
    f = np.float32
    lr, kl, d = f(lr), f(kl), f(d)
    if kl > f(2.0) * d:
        return max(f(lo), lr / f(1.5))
    if kl < f(0.5) * d:
        return min(f(hi), lr * f(1.5))
    return lr


def test_kl_adaptive_learning_rate(L):
    """The device-resident learning rate: bounds and switch-off exactly; the rule applied to the library's own
    approx_kl reproduces the reported rates; the Adam step really uses the reported rate; the rates agree with
    the oracle's on a target its divergences stay clear of; lr_carry continues where the last update stopped."""
    torch = _torch()
    cfg = configs.get_config(0, num_envs=64, horizon=16)
    base = dict(cfg["hp"], epochs=3, seed=21, lr_min=1e-4, lr_max=1.5e-3)
    lr0, n = base["lr"], base["epochs"] * base["minibatches"]

    def run(**kw):
        lrn, ro, params = _setup(L, cfg)
        lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), base["gamma"], base["lam"])
        return lrn, ro, params, lrn.update(dict(base, **kw))

    lrn_off, ro, params, st_off = run()
    assert [s["lr"] for s in st_off] == [float(np.float32(lr0))] * n
    _, _, _, st0 = run(desired_kl=0.0, lr_carry=1)
    assert st0 == st_off                                                       # off: the other fields do nothing
    up = [s["lr"] for s in run(desired_kl=1e9)[3]]
    np.testing.assert_allclose(up, [min(1.5e-3, lr0 * 1.5 ** (k + 1)) for k in range(n)], rtol=1e-6)
    down = [s["lr"] for s in run(desired_kl=1e-12)[3]]
    np.testing.assert_allclose(down, [max(1e-4, lr0 / 1.5 ** (k + 1)) for k in range(n)], rtol=1e-6)

    def own_rule(st, d):
        lr, seq = lr0, []
        for k, s in enumerate(st):                                              # the rule on the library's own numbers, exactly
            lr = _rule32(lr, s["approx_kl"], d, base["lr_min"], base["lr_max"])
            assert s["lr"] == float(lr), (k, s["lr"], lr)
            seq.append(float(lr))
        return seq

    # thresholds inside the spread of the minibatch divergences: the rate moves on some steps and holds on others
    kls = sorted(s["approx_kl"] for s in st_off)
    med = 0.5 * (kls[n // 2 - 1] + kls[n // 2])
    seq_a = own_rule(run(desired_kl=0.5 * med)[3], 0.5 * med)                   # upper threshold 2d at the median
    seq_b = own_rule(run(desired_kl=2.0 * med)[3], 2.0 * med)                   # lower threshold d/2 at the median
    assert len(set(seq_a)) >= 2 and len(set(seq_b)) >= 2
    assert any(x == y for x, y in zip(seq_a, [lr0] + seq_a)) or any(x == y for x, y in zip(seq_b, [lr0] + seq_b))   # a hold

    # against the oracle: a target (picked deterministically) that keeps the oracle's divergences clear of both thresholds
    fr, adv, ret = _oracle_inputs(cfg, ro, lrn_off)
    z = np.zeros_like(params, dtype=np.float64)
    for d in (0.25 * med, 0.2 * med, 0.15 * med, 4.0 * med, 5.0 * med):
        hp = dict(base, desired_kl=float(d))
        with orc.quant(1):
            out = orc.ppo_update(cfg["net"], params, z, z, 0, fr["obs"], fr["proprio"], fr["action"], fr["logp_old"], fr["value"],
                                 adv, ret, hp, update_idx=0)
        margin = min(min(abs(o["approx_kl"] / (2 * d) - 1), abs(o["approx_kl"] / (0.5 * d) - 1)) for o in out["stats"])
        if margin > 0.15:
            break
    else:
        pytest.fail("no target keeps the oracle's divergences clear of the thresholds")
    lrn, _, _, st = run(desired_kl=float(d))
    own_rule(st, d)
    np.testing.assert_allclose([s["lr"] for s in st], [o["lr"] for o in out["stats"]], rtol=1e-6)
    for s, o in zip(st, out["stats"]):
        assert abs(s["approx_kl"] - o["approx_kl"]) <= 0.1 * o["approx_kl"] + 1e-6
    _compare_update(L, cfg, lrn, ro, params, out, st, max(o["lr"] for o in out["stats"]))

    # lr_carry: the next update goes on from the stored rate, or restarts from hp.lr
    last = st[-1]["lr"]
    st2 = lrn.update(dict(base, desired_kl=float(d), lr_carry=1))
    assert st2[0]["lr"] == float(_rule32(last, st2[0]["approx_kl"], d, base["lr_min"], base["lr_max"]))
    st3 = lrn.update(dict(base, desired_kl=float(d), lr_carry=0))
    assert st3[0]["lr"] == float(_rule32(lr0, st3[0]["approx_kl"], d, base["lr_min"], base["lr_max"]))


def test_kl_adaptive_rate_at_the_benchmark_size(L):
    """The schedule in the launch configuration bench.py times (1024 envs x 16 steps, 2 epochs x 4 minibatches of 4096):
    every reported rate follows from the library's own approx_kl by the rule in fp32, the rates stay inside the bounds,
    and the statistics of the first step equal those of the run without the schedule (the loss does not depend on the rate)."""
    torch = _torch()
    cfg = configs.get_config(1)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], seed=11)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    st_off = lrn.update(hp)
    kls = sorted(s["approx_kl"] for s in st_off)
    d = float(kls[len(kls) // 2])                       # upper threshold above, lower threshold below every divergence but the rate still moves
    lrn2, _, _ = _setup(L, cfg)
    lrn2.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    hp2 = dict(hp, desired_kl=0.5 * d, lr_min=1e-5, lr_max=1e-2)
    st = lrn2.update(hp2)
    lr = hp["lr"]
    for k, s in enumerate(st):
        lr = _rule32(lr, s["approx_kl"], 0.5 * d, 1e-5, 1e-2)
        assert s["lr"] == float(lr), (k, s["lr"], lr)
        assert 1e-5 <= s["lr"] <= 1e-2 and s["nonfinite"] == 0
    for f in ("pi_loss", "v_loss", "approx_kl", "total_loss", "grad_norm"):
        assert st[0][f] == st_off[0][f], f
    assert len({s["lr"] for s in st}) >= 2
    assert np.isfinite(lrn2.get_params()).all()


def test_kl_adaptive_rate_is_the_one_adam_uses(L):
    """Single-minibatch updates with a target far above any divergence: each step's rate is 1.5 x the last, and the
    oracle's Adam with the reported rate, applied to the reported gradient, reproduces the parameters."""
    torch = _torch()
    cfg = configs.get_config(0, num_envs=64, horizon=16)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], epochs=1, minibatches=1, seed=3, desired_kl=1e9, lr_min=1e-5, lr_max=1.0, lr_carry=1)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    p = params.astype(np.float64)
    m, v = np.zeros_like(p), np.zeros_like(p)
    for k in (1, 2, 3):
        st = lrn.update(hp)[0]
        assert abs(st["lr"] / (hp["lr"] * 1.5 ** k) - 1) < 1e-6
        g = lrn.get_grads().astype(np.float64)
        orc.adam_step(p, m, v, g, k, lr=st["lr"], beta1=hp["beta1"], beta2=hp["beta2"], eps=hp["adam_eps"])
        got = lrn.get_params().astype(np.float64)
        assert np.abs(got - p).max() <= 1e-6 * max(1.0, np.abs(p).max()) + 2e-3 * st["lr"]
        gm, gv, _, _ = lrn.get_opt_state()
        p, m, v = got.copy(), gm.astype(np.float64), gv.astype(np.float64)


def test_kl_adaptive_argument_errors(L):
    cfg = configs.get_config(0, num_envs=8, horizon=2)
    torch = _torch()
    lrn, ro, params = _setup(L, cfg)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), 0.99, 0.95)
    for bad in (dict(desired_kl=0.01, lr_min=0.0, lr_max=1e-2), dict(desired_kl=0.01, lr_min=1e-2, lr_max=1e-3),
                dict(desired_kl=float("nan")), dict(lr_carry=2), dict(desired_kl=0.01, lr_min=1e-4, lr_max=float("inf"))):
        with pytest.raises(L.LearnerError) as e:
            lrn.update(dict(cfg["hp"], **bad))
        assert e.value.code == L.PPO_EINVAL, bad


@pytest.mark.parametrize("ci,N,T,M", [(0, 2, 2, 4), (0, 3, 1, 1), (1, 1, 1, 1), (1, 5, 3, 3)])
def test_tiny_batches(L, ci, N, T, M):
    """Degenerate sizes: minibatches of one to five samples.  Loss statistics of the first step against the oracle."""
    torch = _torch()
    cfg = configs.get_config(ci, num_envs=N, horizon=T)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], epochs=1, minibatches=M, seed=2)
    lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
    stats = lrn.update(hp)
    assert len(stats) == M and all(s["nonfinite"] == 0 for s in stats)
    fr, adv, ret = _oracle_inputs(cfg, ro, lrn)
    B = N * T // M
    sel = orc.permutation(hp["seed"], 0, 0, N * T)[:B]
    with orc.quant(1):
        qst, _ = orc.ppo_loss_grad(cfg["net"], params, fr["obs"][sel], fr["proprio"][sel], fr["action"][sel], fr["logp_old"][sel],
                                   fr["value"][sel], adv[sel], ret[sel], clip_eps=hp["clip_eps"], vclip_eps=hp["vclip_eps"],
                                   vf_coef=hp["vf_coef"], ent_coef=hp["ent_coef"])
    for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("total_loss", "total")):
        assert abs(stats[0][k_gpu] - qst[k_or]) <= TOL_BF16 * max(abs(qst[k_or]), 1e-2), (k_gpu, stats[0][k_gpu], qst[k_or])


def _stereo_cfg(N, T):
    """The stereo student of config 3 at half resolution (60x80 per view), so that the oracle can
    afford minibatches large enough for a meaningful gradient comparison (two bf16-operand
    implementations that sum in different orders differ at the ulp level, a few ReLU masks flip,
    and on a noise-label batch gradient that shows up as an error ~ 1/sqrt(B))."""
    cfg = configs.get_config(3, num_envs=N, horizon=T)
    cfg["net"].update(in_h=60, in_w=80)
    return cfg


# act_dim 26 = 23 action components + a 3-d auxiliary target (the deployed student's object-position output, Sec. IV-C):
# more outputs of the same linear head under the same mean-squared error
@pytest.mark.parametrize("chunk,act_dim", [(0, 23), (200, 23), (0, 26)])
def test_distill_single_minibatch_gradients(L, chunk, act_dim):
    cfg = _stereo_cfg(128, 4)
    cfg["net"]["act_dim"] = act_dim
    lrn, ro, params = _setup(L, cfg, max_chunk=chunk)
    hp = dict(cfg["hp"], minibatches=1, seed=5)
    st = lrn.distill_update(hp)[0]
    fr = flat_rollout(ro)
    ost, og = orc.distill_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"])
    with orc.quant(1):
        qst, qg = orc.distill_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"])
    for ref in (ost, qst):
        assert abs(st["total_loss"] - ref["total"]) <= TOL_BF16 * abs(ref["total"])
    assert abs(st["grad_norm"] - qst["grad_norm"]) <= TOL_BF16 * qst["grad_norm"]
    errs = per_tensor_errors(cfg["net"], lrn.get_grads(), qg)
    print({k: round(v, 4) for k, v in errs.items()})
    assert max(errs.values()) <= TOL_BF16, errs
    assert max(per_tensor_errors(cfg["net"], lrn.get_grads(), og).values()) <= 0.15


@pytest.mark.parametrize("chunk,aux_dim,aux_coef", [(0, 3, 0.3), (200, 3, 2.0), (0, 1, 0.0)])
def test_distill_weighted_auxiliary_output(L, chunk, aux_dim, aux_coef):
    """The student's auxiliary regression output (last aux_dim head columns, own weight): loss parts and gradient of
    one minibatch against the oracle; a multi-step update; weight 0 leaves the auxiliary columns' head rows without
    gradient; bad arguments."""
    cfg = _stereo_cfg(128, 4)
    cfg["net"]["act_dim"] = 26
    lrn, ro, params = _setup(L, cfg, max_chunk=chunk)
    hp = dict(cfg["hp"], minibatches=1, seed=5, aux_dim=aux_dim, aux_coef=aux_coef)
    st = lrn.distill_update(hp)[0]
    fr = flat_rollout(ro)
    with orc.quant(1):
        qst, qg = orc.distill_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"], aux_dim=aux_dim, aux_coef=aux_coef)
    for k_gpu, k_or in (("pi_loss", "pi_loss"), ("v_loss", "v_loss"), ("total_loss", "total")):
        assert abs(st[k_gpu] - qst[k_or]) <= TOL_BF16 * abs(qst[k_or]), (k_gpu, st[k_gpu], qst[k_or])
    assert abs(st["total_loss"] - (st["pi_loss"] + aux_coef * st["v_loss"])) <= 1e-5 * st["total_loss"]
    assert abs(st["grad_norm"] - qst["grad_norm"]) <= TOL_BF16 * qst["grad_norm"]
    g = lrn.get_grads()
    errs = per_tensor_errors(cfg["net"], g, qg)
    assert max(errs.values()) <= TOL_BF16, errs
    # the plain mean over all columns is a different loss: the option is really on
    with orc.quant(1):
        pst, _ = orc.distill_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"])
    assert abs(pst["total"] - qst["total"]) > 10 * TOL_BF16 * abs(qst["total"]) or aux_coef == 0.0
    if aux_coef == 0.0:
        a, b, shape = synth.param_slices(cfg["net"])["mu.w"]
        hw = g[a:b].reshape(shape)
        assert np.all(hw[26 - aux_dim:] == 0) and np.any(hw[:26 - aux_dim] != 0)
        for bad in (dict(aux_dim=26), dict(aux_dim=-1), dict(aux_dim=2, aux_coef=-1.0), dict(aux_dim=2, aux_coef=float("nan"))):
            with pytest.raises(L.LearnerError) as e:
                lrn.distill_update(dict(hp, **bad))
            assert e.value.code == L.PPO_EINVAL, bad
    else:
        lrn2, _, _ = _setup(L, cfg, max_chunk=chunk)
        hp2 = dict(cfg["hp"], seed=5, aux_dim=aux_dim, aux_coef=aux_coef)
        stats = lrn2.distill_update(hp2)
        z = np.zeros_like(params, dtype=np.float64)
        with orc.quant(1):
            out = orc.distill_update(cfg["net"], params, z, z, 0, fr["obs"], fr["proprio"], fr["action"], hp2, update_idx=0)
        for s, o in zip(stats, out["stats"]):
            assert abs(s["total_loss"] - o["total"]) <= TOL_BF16 * abs(o["total"])
            assert abs(s["v_loss"] - o["v_loss"]) <= TOL_BF16 * abs(o["v_loss"])
        assert rel_l2(lrn2.get_params(), out["params"]) <= TOL_BF16


@pytest.mark.parametrize("h,w", [(44, 72), (52, 100), (30, 48)])
def test_distill_gradients_odd_image_shapes(L, h, w):
    """RGB views whose rows are and are not multiples of 16 bytes (the register-fused, the LDS-fused and the
    implicit-GEMM form of the second layer's backward) and bands that do not divide the image."""
    cfg = configs.get_config(3, num_envs=128, horizon=4)
    cfg["net"].update(in_h=h, in_w=w)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], minibatches=1, seed=5)
    st = lrn.distill_update(hp)[0]
    fr = flat_rollout(ro)
    with orc.quant(1):
        qst, qg = orc.distill_loss_grad(cfg["net"], params, fr["obs"], fr["proprio"], fr["action"])
    assert abs(st["total_loss"] - qst["total"]) <= TOL_BF16 * abs(qst["total"])
    assert abs(st["grad_norm"] - qst["grad_norm"]) <= TOL_BF16 * qst["grad_norm"]
    errs = per_tensor_errors(cfg["net"], lrn.get_grads(), qg)
    assert max(errs.values()) <= TOL_BF16, errs


def test_distill_update_matches_oracle(L):
    cfg = _stereo_cfg(64, 4)
    lrn, ro, params = _setup(L, cfg)
    hp = dict(cfg["hp"], minibatches=2, seed=5)
    stats = lrn.distill_update(hp)
    fr = flat_rollout(ro)
    z = np.zeros_like(params, dtype=np.float64)
    with orc.quant(1):
        out = orc.distill_update(cfg["net"], params, z, z, 0, fr["obs"], fr["proprio"], fr["action"], hp, update_idx=0)
    for k, (s, o) in enumerate(zip(stats, out["stats"])):
        assert abs(s["total_loss"] - o["total"]) <= TOL_BF16 * abs(o["total"])
        assert abs(s["grad_norm"] - o["grad_norm"]) <= (TOL_BF16 if k == 0 else 0.25) * o["grad_norm"]
    assert rel_l2(lrn.get_params(), out["params"]) <= TOL_BF16
    errs = per_tensor_param_errors(cfg["net"], lrn.get_params(), out["params"], len(stats), hp["lr"])
    assert max(errs.values()) <= 2.5 * TOL_BF16, errs


# ------------------------------------------------------------------ host logic on a live context
def test_call_order_and_argument_errors(L):
    torch = _torch()
    cfg = configs.get_config(0, num_envs=8, horizon=3)
    lrn = L.Learner(cfg["net"], 8, 3, "fp32")
    lv = torch.zeros(8, device="cuda")
    with pytest.raises(L.LearnerError) as e:
        lrn.gae(lv, 0.99, 0.95)
    assert e.value.code == L.PPO_ESTATE
    ro = synth.rollout(cfg)
    fill_learner(lrn, cfg, ro)
    with pytest.raises(L.LearnerError) as e:
        lrn.update(dict(cfg["hp"], epochs=1, minibatches=1))
    assert e.value.code == L.PPO_ESTATE
    lrn.gae(lv, 0.99, 0.95)
    with pytest.raises(L.LearnerError) as e:
        lrn.update(dict(cfg["hp"], epochs=1, minibatches=5))
    assert e.value.code == L.PPO_ESHAPE
    with pytest.raises(L.LearnerError) as e:
        lrn.update(dict(cfg["hp"], epochs=1, minibatches=1, lr=float("nan")))
    assert e.value.code == L.PPO_EINVAL
    with pytest.raises(L.LearnerError) as e:
        lrn.distill_update(dict(cfg["hp"], epochs=1, minibatches=1))
    assert e.value.code == L.PPO_ESTATE
    with pytest.raises(L.LearnerError) as e:
        lrn.gae(lv, 1.5, 0.95)
    assert e.value.code == L.PPO_EINVAL


def test_update_is_deterministic_and_resumable(L):
    torch = _torch()
    cfg = configs.get_config(0, num_envs=64, horizon=16)
    hp = dict(cfg["hp"], epochs=2, seed=7)
    runs = []
    for _ in range(2):
        lrn, ro, params = _setup(L, cfg)
        lrn.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
        lrn.update(hp)
        runs.append((lrn.get_params(), lrn.get_opt_state(), lrn))
    np.testing.assert_array_equal(runs[0][0], runs[1][0])
    # checkpoint -> fresh context -> the next update is bit-identical
    a = runs[0][2]
    b = L.Learner(cfg["net"], cfg["num_envs"], cfg["horizon"], cfg["obs_dtype"])
    b.set_params(runs[0][0])
    m, v, step, upd = runs[0][1]
    b.set_opt_state(m, v, step, upd)
    ro = synth.rollout(cfg)
    fill_learner(b, cfg, ro)
    for x in (a, b):
        x.gae(torch.from_numpy(ro["last_value"]).cuda(), hp["gamma"], hp["lam"])
        x.update(hp)
    np.testing.assert_array_equal(a.get_params(), b.get_params())


def test_resume_carries_the_adaptive_rate(L):
    """Checkpoint of a context that runs the KL-adaptive rate with lr_carry: parameters, optimiser state AND the rate
    the last update ended with; the resumed context's next update is bit-identical, and without the rate it is not."""
    torch = _torch()
    cfg = configs.get_config(0, num_envs=64, horizon=16)
    hp = dict(cfg["hp"], epochs=3, seed=7, desired_kl=1e-6, lr_min=1e-5, lr_max=1e-2, lr_carry=1)   # every divergence is above 2e-6: the rate falls
    a, ro, params = _setup(L, cfg)
    lv = torch.from_numpy(ro["last_value"]).cuda()
    assert a.get_adaptive_lr() == (0.0, False)
    a.gae(lv, hp["gamma"], hp["lam"])
    st = a.update(hp)
    lr, live = a.get_adaptive_lr()
    assert live and lr == st[-1]["lr"] and lr < hp["lr"]
    ckpt = (a.get_params(), a.get_opt_state(), lr)
    outs = []
    for with_rate in (True, False):
        b = L.Learner(cfg["net"], cfg["num_envs"], cfg["horizon"], cfg["obs_dtype"])
        b.set_params(ckpt[0])
        b.set_opt_state(*ckpt[1])
        if with_rate:
            b.set_adaptive_lr(ckpt[2])
        fill_learner(b, cfg, ro)
        b.gae(lv, hp["gamma"], hp["lam"])
        outs.append((b.update(hp), b.get_params()))
    a.update(hp)
    np.testing.assert_array_equal(a.get_params(), outs[0][1])
    assert outs[0][0][0]["lr"] != outs[1][0][0]["lr"] and not np.array_equal(outs[0][1], outs[1][1])
    with pytest.raises(L.LearnerError) as e:
        a.set_adaptive_lr(-1.0)
    assert e.value.code == L.PPO_EINVAL
    a.set_adaptive_lr(0.0, live=False)
    assert a.get_adaptive_lr() == (0.0, False)
