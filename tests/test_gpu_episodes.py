"""k episodes per environment copy (the auto-reset environment wrapper of the paper's Sec. 3.1) on
every rollout kernel, against the CPU checker, which runs them one after the other."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, Workload, make_inputs
from gpu_util import assert_params_close, compare_rollout, dev, noise_to_device, run_rollout, probe_rollout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import paper_2501_15129_amd as pkg
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pkg


CASES = [
    (replace(CONFIGS[0], name="cfg0-k3", episodes=3), "wave_reg"),
    (replace(CONFIGS[1], name="cfg1-k2-T120", episodes=2, horizon=120, pop=8, envs=5), "wave_reg"),
    (Workload("odd-k4", pop=6, envs=3, horizon=50, obs=13, hid=29, act=7, dtype=0, noise_dtype=0, seed=51, episodes=4), "wave_reg"),
    (Workload("wide-k2", pop=4, envs=2, horizon=30, obs=70, hid=100, act=9, dtype=0, noise_dtype=0, seed=57, episodes=2), "wave_lds_f32"),
    (Workload("odd-k2-bf16", pop=6, envs=3, horizon=50, obs=13, hid=29, act=7, dtype=1, noise_dtype=1, seed=52, episodes=2), "wave_reg_bf16"),
    (Workload("wide-k2-bf16", pop=4, envs=2, horizon=30, obs=70, hid=100, act=9, dtype=1, noise_dtype=1, seed=58, episodes=2), "wave_lds_bf16"),
    (Workload("mfma32-k5", pop=4, envs=5, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=53, episodes=5), "mfma"),   # 25 columns: ragged second block
    (Workload("mfma32-narrow-k2", pop=4, envs=2, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=54, episodes=2), "mfma"),
    (Workload("mfma256-k4", pop=4, envs=4, horizon=16, obs=244, hid=256, act=17, dtype=1, noise_dtype=1, seed=55, episodes=4,
              done_thresh=math.inf), "mfma"),
    (Workload("depth3-k2", pop=6, envs=2, horizon=40, obs=11, hid=24, act=3, dtype=0, noise_dtype=0, seed=56, episodes=2, num_hidden=3), "wave_lds_f32"),
]


@pytest.mark.parametrize("w,kernel", CASES, ids=lambda x: x.name if isinstance(x, Workload) else x)
def test_rollout_episodes_per_env(es, w, kernel):
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    assert kernel in ctx.rollout_kernel and ctx.episodes == w.envs * w.episodes
    eps = oracle.sample_population(w, 1)
    got = run_rollout(ctx, w, 1, theta, noise_to_device(ctx, eps), a_mat, b_mat)
    assert got[0].shape == (w.pop, w.envs * w.episodes)
    ref = oracle.rollout(w, 1, theta, eps, a_mat, b_mat)
    probe = probe_rollout(w, 1, theta, eps, a_mat, b_mat, ref=ref)
    flips, worst, sens, chaotic = compare_rollout(w, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens}")
    assert not chaotic


def test_generation_with_episodes_per_env(es):
    """sample -> rollout -> rank -> update with 3 episodes per copy: fitness is the mean over all 12."""
    w = replace(CONFIGS[0], name="cfg0-k3-gen", episodes=3, done_thresh=math.inf)
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    noise = ctx.alloc_noise()
    ctx.sample_population(0, noise)
    eps = oracle.sample_population(w, 0)
    assert np.array_equal(noise.float().cpu().numpy()[:, :w.n_params], eps)
    ret, ln, fit = run_rollout(ctx, w, 0, theta, noise, a_mat, b_mat)
    r_ret, r_len, r_fit, _ = oracle.rollout(w, 0, theta, eps, a_mat, b_mat)
    np.testing.assert_allclose(fit, r_fit, rtol=1e-4)
    fit_d, rank_d, shaped_d = dev(fit), torch.empty(w.pop, dtype=torch.int32, device="cuda"), torch.empty(w.pop, device="cuda")
    ctx.rank(fit_d, rank_d, shaped_d)
    theta_d, m_d, v_d = dev(theta), torch.zeros(w.n_params, device="cuda"), torch.zeros(w.n_params, device="cuda")
    grad_d = torch.empty(w.n_params, device="cuda")
    ctx.update(1, noise, shaped_d, theta_d, m_d, v_d, grad_d, ctx.alloc_workspace())
    torch.cuda.synchronize()
    r_rank, r_shaped = oracle.rank(fit)                      # the kernel's own fitness: ranks are bit-exact
    assert np.array_equal(rank_d.cpu().numpy(), r_rank)
    zeros = np.zeros(w.n_params, dtype=np.float32)
    t2, m2, v2, _ = oracle.update(w, 1, eps, r_shaped, theta, zeros, zeros)
    assert_params_close(theta_d.cpu().numpy(), t2, "theta")


@pytest.mark.parametrize("idx", [3, 4])
def test_full_size_configs_with_four_episodes_per_env(es, idx):
    """configs[3] / [4] at full population with k = 4 (config 4 then fills all 16 matrix-core columns), in the
    launch configuration of `bench.py --episodes-per-env 4`.  At the long horizon the outputs are checked for
    the properties that hold at any size; the checker recomputes sampled mirrored pairs at a horizon short
    enough for bf16 trajectories not to have diverged (the per-step code path is the same for every step)."""
    w = replace(CONFIGS[idx], name=f"cfg{idx}-k4", episodes=4, horizon=200, done_thresh=math.inf)
    a_mat, b_mat, theta = make_inputs(w)
    ctx = es.EsContext(w)
    noise = ctx.alloc_noise()
    ctx.sample_population(0, noise)
    ret, ln, fit = run_rollout(ctx, w, 0, theta, noise, a_mat, b_mat)
    assert ret.shape == (w.pop, 4 * w.envs) and np.all(ln == w.horizon) and np.all(np.isfinite(ret))
    assert np.allclose(fit, ret.astype(np.float64).mean(axis=1), rtol=1e-5, atol=1e-5)
    assert np.all(np.abs(ret) <= w.horizon * (1.0 + w.act_cost * w.act))         # |r_t| <= 1 + c * n_a
    short = replace(w, name=f"{w.name}-short", horizon=40 if idx == 3 else 16)
    ctx_s = es.EsContext(short)
    got = run_rollout(ctx_s, short, 0, theta, noise, a_mat, b_mat)
    del noise
    torch.cuda.empty_cache()
    rng = np.random.default_rng(idx)
    rows = np.unique(np.concatenate([[0, w.noise_rows - 1], rng.integers(0, w.noise_rows, size=2)]))
    refs, probes, subs = [], [], []
    for j in rows:
        eps_j = oracle.sample_population(short, 0, rows=(j, j + 1))
        ind = (2 * j, 2 * j + 2)
        refs.append(oracle.rollout(short, 0, theta, eps_j, a_mat, b_mat, individuals=ind, noise_row0=j))
        probes.append(probe_rollout(short, 0, theta, eps_j, a_mat, b_mat, individuals=ind, noise_row0=j, ref=refs[-1]))
        subs.append(tuple(x[ind[0]:ind[1]] for x in got))
    cat = lambda parts: tuple(np.concatenate([p[k] for p in parts]) for k in range(len(parts[0])))
    flips, worst, sens, chaotic = compare_rollout(short, cat(subs), cat(refs), short.name, cat(probes))
    print(f"[{short.name}] rows {rows.tolist()}: worst {worst:.2e} sensitive {sens} of {cat(refs)[0].size}")
    assert not chaotic
