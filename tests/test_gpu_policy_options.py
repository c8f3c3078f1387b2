"""Policy options of the paper's EA experiments (App. B): ReLU hidden layers and small [16, 16]
networks (Sec. 5.2), on every rollout kernel, against the CPU checker."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, Workload, make_inputs
from gpu_util import compare_rollout, noise_to_device, run_rollout, probe_rollout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import paper_2501_15129_amd as pkg
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pkg


def _case(es, w, gen=1, expect_kernel=None):
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    if expect_kernel:
        assert expect_kernel in ctx.rollout_kernel, ctx.rollout_kernel
    eps = oracle.sample_population(w, gen)
    got = run_rollout(ctx, w, gen, theta, noise_to_device(ctx, eps), a_mat, b_mat)
    ref = oracle.rollout(w, gen, theta, eps, a_mat, b_mat)
    probe = probe_rollout(w, gen, theta, eps, a_mat, b_mat, ref=ref)
    flips, worst, sens, chaotic = compare_rollout(w, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens} chaotic {chaotic}")
    assert not chaotic
    return got


RELU_CASES = [
    (Workload("relu-odd", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=22, hidden_act=1), "wave_reg"),
    (Workload("relu-wide", pop=4, envs=2, horizon=40, obs=70, hid=100, act=9, dtype=0, noise_dtype=0, seed=24, hidden_act=1), "wave_lds_f32"),
    (Workload("relu-odd-bf16", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=1, noise_dtype=1, seed=22, hidden_act=1), "wave_reg_bf16"),
    (Workload("relu-wide-bf16", pop=4, envs=2, horizon=40, obs=70, hid=100, act=9, dtype=1, noise_dtype=1, seed=25, hidden_act=1), "wave_lds_bf16"),
    (Workload("relu-linear-out", pop=6, envs=3, horizon=40, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=23, hidden_act=1, out_tanh=0), "wave_reg"),
    (replace(CONFIGS[0], name="relu-cfg0", hidden_act=1), "wave_reg"),
    (replace(CONFIGS[1], name="relu-cfg1-T150", hidden_act=1, horizon=150), "wave_reg"),
    (Workload("relu-mfma32", pop=6, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=31, hidden_act=1), "mfma"),
    (Workload("relu-mfma32-narrow", pop=4, envs=3, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=32, hidden_act=1), "mfma"),
    (Workload("relu-mfma64", pop=4, envs=16, horizon=30, obs=60, hid=256, act=10, dtype=1, noise_dtype=1, seed=35, hidden_act=1), "mfma"),
    (Workload("relu-mfma128", pop=4, envs=16, horizon=30, obs=100, hid=200, act=20, dtype=1, noise_dtype=1, seed=33, hidden_act=1), "mfma"),
    (Workload("relu-mfma256", pop=4, envs=4, horizon=16, obs=244, hid=256, act=17, dtype=1, noise_dtype=1, seed=34, hidden_act=1,
              done_thresh=math.inf), "mfma"),
]


@pytest.mark.parametrize("w,kernel", RELU_CASES, ids=lambda x: x.name if isinstance(x, Workload) else x)
def test_rollout_relu_hidden_layers(es, w, kernel):
    _case(es, w, expect_kernel=kernel)


@pytest.mark.parametrize("hidden_act", [0, 1])
@pytest.mark.parametrize("dtype", [0, 1])
def test_rollout_small_16_16_network(es, hidden_act, dtype):
    """The [16, 16] policies of the paper's Sec. 5.2 comparison."""
    w = Workload(f"net16-a{hidden_act}-d{dtype}", pop=12, envs=4, horizon=80, obs=17, hid=16, act=6, dtype=dtype,
                 noise_dtype=dtype, seed=40 + hidden_act, hidden_act=hidden_act)
    _case(es, w)


@pytest.mark.parametrize("idx", [3, 4])
def test_rollout_relu_full_size_bf16_configs(es, idx):
    """configs[3] and [4] with ReLU hidden layers, full population, in the launch configuration of
    `bench.py --hidden-act relu`; the checker recomputes sampled mirrored pairs."""
    w = replace(CONFIGS[idx], name=f"cfg{idx}-relu", hidden_act=1)
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    noise = ctx.alloc_noise()
    ctx.sample_population(0, noise)
    got = run_rollout(ctx, w, 0, theta, noise, a_mat, b_mat)
    del noise
    torch.cuda.empty_cache()
    assert np.all(np.isfinite(got[0])) and np.all(got[1] >= 1) and np.all(got[1] <= w.horizon)
    refs, probes, subs = [], [], []
    for j in (0, 1, w.pop // 4, w.pop // 2 - 1):
        eps = oracle.sample_population(w, 0, rows=(j, j + 1))
        ind = (2 * j, 2 * j + 2)
        refs.append(oracle.rollout(w, 0, theta, eps, a_mat, b_mat, individuals=ind, noise_row0=j))
        probes.append(probe_rollout(w, 0, theta, eps, a_mat, b_mat, individuals=ind, noise_row0=j, ref=refs[-1]))
        subs.append(tuple(x[ind[0]:ind[1]] for x in got))
    cat = lambda parts: tuple(np.concatenate([p[k] for p in parts]) for k in range(len(parts[0])))
    flips, worst, sens, chaotic = compare_rollout(w, cat(subs), cat(refs), w.name, cat(probes))
    print(f"[{w.name}] worst {worst:.2e} flips {flips} sensitive {sens} chaotic {chaotic}")
    assert not chaotic


# ---- frozen observation normalisation (paper App. B) ----
def _stats(w, seed=9):
    rng = np.random.default_rng(seed)
    mean = (rng.standard_normal(w.obs) * 0.05).astype(np.float32)
    inv = (1.0 / (0.33 + rng.random(w.obs) * 0.67)).astype(np.float32)      # standard deviations of 0.33 .. 1
    return mean, inv


NORM_CASES = [
    Workload("norm-odd", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=22),
    Workload("norm-odd-bf16", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=1, noise_dtype=1, seed=22),
    replace(CONFIGS[0], name="norm-cfg0"),
    replace(CONFIGS[1], name="norm-cfg1-T40-relu", horizon=40, hidden_act=1),
    Workload("norm-mfma32", pop=6, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=31),
    Workload("norm-mfma32-narrow-relu", pop=4, envs=3, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=32, hidden_act=1),
    Workload("norm-mfma64", pop=4, envs=16, horizon=30, obs=60, hid=256, act=10, dtype=1, noise_dtype=1, seed=35),
    Workload("norm-mfma128", pop=4, envs=16, horizon=30, obs=100, hid=200, act=20, dtype=1, noise_dtype=1, seed=33),
    Workload("norm-mfma256", pop=4, envs=4, horizon=16, obs=244, hid=256, act=17, dtype=1, noise_dtype=1, seed=34, done_thresh=math.inf),
    Workload("norm-mfma256-wide-regen", pop=4, envs=16, horizon=16, obs=244, hid=256, act=17, dtype=1, noise_dtype=3, seed=36,
             done_thresh=math.inf),
]


@pytest.mark.parametrize("w", NORM_CASES, ids=lambda w: w.name)
def test_rollout_with_observation_statistics(es, w):
    from gpu_util import dev
    ws = replace(w, noise_dtype=w.noise_dtype & 1)
    a_mat, b_mat, theta = make_inputs(w)
    mean, inv = _stats(w)
    ctx = es.EsContext(w)
    eps = oracle.sample_population(ws, 1)
    noise = None if ctx.noise_regenerated else noise_to_device(ctx, eps)
    plain = run_rollout(ctx, w, 1, theta, noise, a_mat, b_mat)
    ctx.set_obs_norm(dev(mean), dev(inv))
    got = run_rollout(ctx, w, 1, theta, noise, a_mat, b_mat)
    ref = oracle.rollout(ws, 1, theta, eps, a_mat, b_mat, obs_norm=(mean, inv))
    probe = probe_rollout(ws, 1, theta, eps, a_mat, b_mat, obs_norm=(mean, inv), ref=ref)
    flips, worst, sens, chaotic = compare_rollout(ws, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens} chaotic {chaotic}")
    assert not chaotic
    assert np.max(np.abs(got[0] - plain[0])) > 1e-3                     # the statistics were used
    # identity statistics and switching off both give back the plain result, bit for bit
    ctx.set_obs_norm(dev(np.zeros(w.obs, np.float32)), dev(np.ones(w.obs, np.float32)))
    ident = run_rollout(ctx, w, 1, theta, noise, a_mat, b_mat)
    ctx.set_obs_norm(None, None)
    off = run_rollout(ctx, w, 1, theta, noise, a_mat, b_mat)
    for x, y, z in zip(plain, ident, off):
        assert np.array_equal(x.view(np.uint32), y.view(np.uint32)) and np.array_equal(x.view(np.uint32), z.view(np.uint32))


def test_obs_norm_needs_both_arrays(es):
    from gpu_util import dev
    ctx = es.EsContext(CONFIGS[0])
    with pytest.raises(es.EsError):
        ctx.set_obs_norm(dev(np.zeros(CONFIGS[0].obs, np.float32)), None)


# ---- m hidden layers (paper Sec. 5.1 varies the depth of the policy) ----
DEPTH_CASES = [
    Workload("depth1", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=61, num_hidden=1),
    Workload("depth3", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=62, num_hidden=3),
    Workload("depth4-relu-bf16", pop=6, envs=3, horizon=40, obs=13, hid=29, act=7, dtype=1, noise_dtype=1, seed=63, num_hidden=4,
             hidden_act=1),
    Workload("depth3-regen-noanti", pop=7, envs=2, horizon=40, obs=17, hid=64, act=6, dtype=0, noise_dtype=2, seed=64, num_hidden=3,
             antithetic=0),
    Workload("depth1-cfg1-shape", pop=6, envs=4, horizon=50, obs=17, hid=64, act=6, dtype=0, noise_dtype=0, seed=65, num_hidden=1),
    Workload("depth3-hid160-act20-bf16", pop=2, envs=2, horizon=12, obs=8, hid=160, act=20, dtype=1, noise_dtype=1, seed=66, num_hidden=3,
             done_thresh=math.inf),
]


@pytest.mark.parametrize("w", DEPTH_CASES, ids=lambda w: w.name)
def test_rollout_other_depths(es, w):
    ws = replace(w, noise_dtype=w.noise_dtype & 1)
    a_mat, b_mat, theta = make_inputs(w)
    theta = (theta + np.random.default_rng(w.seed).standard_normal(theta.size) * 0.02).astype(np.float32)   # non-zero biases
    ctx = es.EsContext(w)
    assert ctx.param_count == w.n_params and "wave_lds" in ctx.rollout_kernel
    eps = oracle.sample_population(ws, 2)
    noise = None if ctx.noise_regenerated else noise_to_device(ctx, eps)
    got = run_rollout(ctx, w, 2, theta, noise, a_mat, b_mat)
    ref = oracle.rollout(ws, 2, theta, eps, a_mat, b_mat)
    probe = probe_rollout(ws, 2, theta, eps, a_mat, b_mat, ref=ref)
    flips, worst, sens, chaotic = compare_rollout(ws, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} D={ctx.param_count} worst {worst:.2e} flips {flips} sensitive {sens}")
    assert not chaotic


# one, three and four hidden layers of the paper's width (256) in bf16: the matrix-core kernel skips the second layer's
# phase, or keeps the extra layers in registers
DEEP_MFMA_CASES = [
    Workload("deep3-obs8", pop=4, envs=16, horizon=40, obs=8, hid=256, act=2, dtype=1, noise_dtype=1, seed=71, num_hidden=3),
    Workload("deep4-obs8", pop=4, envs=16, horizon=40, obs=8, hid=256, act=2, dtype=1, noise_dtype=1, seed=72, num_hidden=4),
    Workload("deep3-narrow-relu", pop=4, envs=3, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=73, num_hidden=3,
             hidden_act=1),
    Workload("deep4-narrow", pop=4, envs=1, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=74, num_hidden=4),
    Workload("deep3-obs60-hid200", pop=4, envs=20, horizon=30, obs=60, hid=200, act=10, dtype=1, noise_dtype=1, seed=75, num_hidden=3),
    Workload("deep4-obs60-relu", pop=4, envs=16, horizon=30, obs=60, hid=256, act=10, dtype=1, noise_dtype=1, seed=76, num_hidden=4,
             hidden_act=1),
    Workload("one-layer-obs8", pop=4, envs=16, horizon=40, obs=8, hid=256, act=2, dtype=1, noise_dtype=1, seed=61, num_hidden=1),
    Workload("one-layer-narrow-relu", pop=4, envs=3, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=62, num_hidden=1,
             hidden_act=1),
    Workload("one-layer-obs60-hid200", pop=4, envs=20, horizon=30, obs=60, hid=200, act=10, dtype=1, noise_dtype=1, seed=63, num_hidden=1),
    Workload("one-layer-obs60-narrow-linear", pop=4, envs=2, horizon=30, obs=60, hid=256, act=16, dtype=1, noise_dtype=1, seed=64, num_hidden=1,
             out_tanh=0),
    Workload("deep3-regen-linear-out", pop=5, envs=4, horizon=30, obs=17, hid=256, act=6, dtype=1, noise_dtype=3, seed=77, num_hidden=3,
             antithetic=0, out_tanh=0),
]


@pytest.mark.parametrize("w", DEEP_MFMA_CASES, ids=lambda w: w.name)
def test_rollout_deep_policies_on_the_matrix_core_kernel(es, w):
    ws = replace(w, noise_dtype=w.noise_dtype & 1)
    a_mat, b_mat, theta = make_inputs(w)
    theta = (theta + np.random.default_rng(w.seed).standard_normal(theta.size) * 0.02).astype(np.float32)   # non-zero biases
    ctx = es.EsContext(w)
    assert ctx.param_count == w.n_params and "mfma" in ctx.rollout_kernel and f"depth{w.num_hidden}" in ctx.rollout_kernel
    eps = oracle.sample_population(ws, 2)
    noise = None if ctx.noise_regenerated else noise_to_device(ctx, eps)
    got = run_rollout(ctx, w, 2, theta, noise, a_mat, b_mat)
    ref = oracle.rollout(ws, 2, theta, eps, a_mat, b_mat)
    probe = probe_rollout(ws, 2, theta, eps, a_mat, b_mat, ref=ref)
    flips, worst, sens, chaotic = compare_rollout(ws, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} D={ctx.param_count} worst {worst:.2e} flips {flips} sensitive {sens}")
    assert not chaotic


def test_deep_policy_with_obs_norm_on_the_matrix_core_kernel(es):
    from gpu_util import dev
    w = Workload("deep3-norm", pop=4, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=78, num_hidden=3)
    a_mat, b_mat, theta = make_inputs(w)
    rng = np.random.default_rng(78)
    mean = (rng.standard_normal(w.obs) * 0.05).astype(np.float32)
    inv = (1.0 / (0.33 + rng.random(w.obs) * 0.67)).astype(np.float32)
    ctx = es.EsContext(w)
    mean_d, inv_d = dev(mean), dev(inv)
    ctx.set_obs_norm(mean_d, inv_d)
    eps = oracle.sample_population(w, 1)
    got = run_rollout(ctx, w, 1, theta, noise_to_device(ctx, eps), a_mat, b_mat)
    ref = oracle.rollout(w, 1, theta, eps, a_mat, b_mat, obs_norm=(mean, inv))
    probe = probe_rollout(w, 1, theta, eps, a_mat, b_mat, obs_norm=(mean, inv), ref=ref)
    flips, worst, sens, chaotic = compare_rollout(w, got, ref, w.name, probe)
    assert not chaotic


def test_depth_the_register_file_cannot_hold_is_refused(es):
    w = Workload("deep5", pop=4, envs=16, horizon=10, obs=8, hid=256, act=2, dtype=1, noise_dtype=1, seed=79, num_hidden=5)
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    with pytest.raises(es.EsError, match="exceed the LDS"):
        run_rollout(ctx, w, 0, theta, ctx.alloc_noise(), a_mat, b_mat)


def test_generation_with_three_hidden_layers(es):
    """One whole generation at depth 3 through the four calls (the update runs over the longer parameter vector)."""
    from gpu_util import assert_params_close, dev
    w = Workload("depth3-gen", pop=16, envs=2, horizon=30, obs=8, hid=48, act=2, dtype=0, noise_dtype=0, seed=67, num_hidden=3)
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    d = ctx.param_count
    assert d == (8 + 1) * 48 + 2 * 49 * 48 + 49 * 2
    noise, ws = ctx.alloc_noise(), ctx.alloc_workspace()
    th, m, v = dev(theta), torch.zeros(d, device="cuda"), torch.zeros(d, device="cuda")
    ret = torch.empty((w.pop, w.envs), device="cuda")
    ln = torch.empty((w.pop, w.envs), dtype=torch.int32, device="cuda")
    fit = torch.empty(w.pop, device="cuda")
    rk = torch.empty(w.pop, dtype=torch.int32, device="cuda")
    sh = torch.empty(w.pop, device="cuda")
    ctx.sample_population(0, noise)
    ctx.rollout(0, th, noise, dev(a_mat), dev(b_mat), ret, ln, fit, ws)
    ctx.rank(fit, rk, sh)
    ctx.update(1, noise, sh, th, m, v, None, ws)
    torch.cuda.synchronize()
    eps = oracle.sample_population(w, 0)
    assert np.array_equal(noise[:, :d].cpu().numpy().view(np.uint32), eps.view(np.uint32))
    _, _, f_ref, _ = oracle.rollout(w, 0, theta, eps, a_mat, b_mat)
    f_gpu = fit.cpu().numpy()
    assert np.max(np.abs(f_gpu - f_ref) / np.maximum(np.abs(f_ref), 1e-3)) <= 1e-4
    r_rank, r_shaped = oracle.rank(f_gpu)
    assert np.array_equal(rk.cpu().numpy(), r_rank)
    want = oracle.update(w, 1, eps, r_shaped, theta, np.zeros(d, np.float32), np.zeros(d, np.float32))
    assert_params_close(th.cpu().numpy(), want[0], "depth-3 theta")
