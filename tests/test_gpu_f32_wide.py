"""Binary32 policies at the paper's width (Sec. 5.1: hidden layers of 256 units) on the fp32 matrix-core
kernel, against the CPU checker: shapes across its range (65..256 hidden units, obs <= 64, act <= 16), both
activations, observation statistics, every noise mode, several passes of 16 copies, degenerate cases."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import Workload, make_inputs
from gpu_util import compare_rollout, dev, noise_to_device, probe_rollout, run_rollout

pytestmark = pytest.mark.gpu

BASE = Workload("f32w", pop=6, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=0, noise_dtype=0, seed=71)


@pytest.fixture(scope="module")
def es():
    import paper_2501_15129_amd as pkg
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pkg


def _case(es, w, gen=1, obs_norm=None):
    a_mat, b_mat, theta = make_inputs(w)
    theta = (theta + np.random.default_rng(w.seed).standard_normal(theta.size) * 0.02).astype(np.float32)     # non-zero biases
    ctx = es.EsContext(w)
    assert "mfma_reg_f32" in ctx.rollout_kernel, ctx.rollout_kernel
    keep = None
    if obs_norm is not None:
        keep = (dev(obs_norm[0]), dev(obs_norm[1]))
        ctx.set_obs_norm(*keep)
    ws = replace(w, noise_dtype=w.noise_dtype & 1)
    if ctx.noise_table:
        noise = ctx.alloc_noise()
        ctx.build_noise_table(noise)
        ctx.sample_population(gen, noise)
        eps = oracle.table_rows(w, gen, w.noise_table_len, ctx.noise_ld, w.noise_dtype == 5)
    else:
        eps = oracle.sample_population(ws, gen)
        noise = None if ctx.noise_regenerated else noise_to_device(ctx, eps)
    got = run_rollout(ctx, w, gen, theta, noise, a_mat, b_mat)
    ref = oracle.rollout(ws, gen, theta, eps, a_mat, b_mat, obs_norm=obs_norm)
    probe = probe_rollout(ws, gen, theta, eps, a_mat, b_mat, ref=ref, obs_norm=obs_norm)
    flips, worst, sens, chaotic = compare_rollout(ws, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens}")
    assert not chaotic
    return got


@pytest.mark.parametrize("w", [
    BASE,
    replace(BASE, name="f32w-paper-8-256-2-E1", obs=8, act=2, envs=1, horizon=60),
    replace(BASE, name="f32w-60-200-10-E5-relu", obs=60, hid=200, act=10, envs=5, hidden_act=1),
    replace(BASE, name="f32w-33-65-16-E21", obs=33, hid=65, act=16, envs=21, horizon=25),
    replace(BASE, name="f32w-64-256-1-linear", obs=64, act=1, envs=3, out_tanh=0),
    replace(BASE, name="f32w-1-129-3-noanti", obs=1, hid=129, act=3, envs=4, antithetic=0, pop=5),
    replace(BASE, name="f32w-fixedlen", done_thresh=math.inf, horizon=80),
    replace(BASE, name="f32w-T1", horizon=1),
    replace(BASE, name="f32w-len1", done_thresh=1e-6),
    replace(BASE, name="f32w-bf16noise", noise_dtype=1),
    replace(BASE, name="f32w-regen", noise_dtype=2, envs=4),
    replace(BASE, name="f32w-table", noise_dtype=4, noise_table_len=1 << 18, envs=4),
    replace(BASE, name="f32w-k3", envs=3, episodes=3),
    replace(BASE, name="f32w-N300", pop=300, envs=2, horizon=5),
    # the four-copy variant (4x4x1 matrix-core shape, up to eight copies per individual): every observation width class,
    # one and two passes, ragged last pass, several episodes per copy, termination inside an episode, bf16 noise
    replace(BASE, name="f32n-16-256-8-E4", obs=16, envs=4, horizon=50),
    replace(BASE, name="f32n-17-130-5-E8", obs=17, hid=130, act=5, envs=8),
    replace(BASE, name="f32n-32-256-16-E7", obs=32, act=16, envs=7),
    replace(BASE, name="f32n-64-256-16-E6-relu", obs=64, act=16, envs=6, hidden_act=1),
    replace(BASE, name="f32n-48-255-9-k2", obs=48, hid=255, act=9, envs=3, episodes=2),
    replace(BASE, name="f32n-len1", envs=4, done_thresh=1e-6),
    replace(BASE, name="f32n-T1", envs=2, horizon=1),
    replace(BASE, name="f32n-fixedlen-bf16noise", envs=4, done_thresh=math.inf, horizon=80, noise_dtype=1),
    replace(BASE, name="f32n-table-bf16", noise_dtype=5, noise_table_len=1 << 18, envs=3),
    replace(BASE, name="f32n-regen-rounded", noise_dtype=3, envs=5),
    # one hidden layer (the paper's depth sweep): the four-copy kernel whatever the number of copies
    replace(BASE, name="f32n-depth1-paper-8-256-2-E1", obs=8, act=2, envs=1, horizon=60, num_hidden=1),
    replace(BASE, name="f32n-depth1-40-200-11-E16-relu", obs=40, hid=200, act=11, num_hidden=1, hidden_act=1),
    replace(BASE, name="f32n-depth1-64-129-16-E6-fixedlen", obs=64, hid=129, act=16, envs=6, num_hidden=1, done_thresh=math.inf),
], ids=lambda w: w.name)
def test_rollout_f32_wide(es, w):
    _case(es, w)


def test_four_copy_variant_is_chosen_up_to_eight_copies(es):
    for envs, episodes, narrow in ((1, 1, True), (4, 2, True), (8, 1, True), (3, 3, False), (16, 1, False)):
        ctx = es.EsContext(replace(BASE, envs=envs, episodes=episodes))
        assert ("copies4" in ctx.rollout_kernel) == narrow, (envs, episodes, ctx.rollout_kernel)
    ctx = es.EsContext(replace(BASE, num_hidden=1))
    assert "copies4" in ctx.rollout_kernel and "depth1" in ctx.rollout_kernel, ctx.rollout_kernel


def test_rollout_f32_wide_with_observation_statistics(es):
    for w in (replace(BASE, name="f32w-norm"), replace(BASE, name="f32w-norm-60-relu", obs=60, hid=160, act=5, hidden_act=1),
              replace(BASE, name="f32n-norm", envs=4), replace(BASE, name="f32n-norm-60-relu-E5", obs=60, hid=160, act=5, hidden_act=1, envs=5)):
        rng = np.random.default_rng(w.seed)
        mean = (rng.standard_normal(w.obs) * 0.05).astype(np.float32)
        inv = (1.0 / (0.33 + rng.random(w.obs) * 0.67)).astype(np.float32)
        _case(es, w, obs_norm=(mean, inv))


def test_rollout_f32_wide_sigma_zero_and_rerun(es):
    got = _case(es, replace(BASE, name="f32w-sigma0", sigma=0.0))
    assert np.all(got[2].view(np.uint32) == got[2].view(np.uint32)[0])
    for w in (BASE, replace(BASE, name="f32n-rerun", envs=4), replace(BASE, name="f32n-rerun-two-passes", obs=50, envs=7)):
        a_mat, b_mat, theta = make_inputs(w)
        ctx = es.EsContext(w)
        nd = noise_to_device(ctx, oracle.sample_population(w, 0))
        a = run_rollout(ctx, w, 0, theta, nd, a_mat, b_mat)
        b = run_rollout(ctx, w, 0, theta, nd, a_mat, b_mat)
        for x, y in zip(a, b):
            assert np.array_equal(x.view(np.uint32), y.view(np.uint32)), w.name
    got = _case(es, replace(BASE, name="f32n-sigma0", sigma=0.0, envs=4))
    assert np.all(got[2].view(np.uint32) == got[2].view(np.uint32)[0])


def test_paper_base_shape_contractive_full_horizon_strict(es):
    """The base configuration of the paper's timing experiment (Sec. 5.1: two hidden layers of 256, population 128, one
    episode, T = 1000) at Swimmer's widths in binary32, on the contractive variant of the synthetic environment: every
    episode within 1e-4 at the full horizon."""
    w = Workload("paper-base-f32", pop=128, envs=1, horizon=1000, obs=8, hid=256, act=2, dtype=0, noise_dtype=0, seed=5).contractive()
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    eps = oracle.sample_population(w, 0)
    got = run_rollout(ctx, w, 0, theta, noise_to_device(ctx, eps), a_mat, b_mat)
    ref = oracle.rollout(w, 0, theta, eps, a_mat, b_mat)
    probe = probe_rollout(w, 0, theta, eps, a_mat, b_mat, ref=ref, probes=1)
    flips, worst, sens, chaotic = compare_rollout(w, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} sensitive {sens}")
    assert not chaotic and compare_rollout.last_excused == 0 and np.all(got[1] == w.horizon)
