"""bf16 policies on a binary32 environment (es_config.env_dtype = 1): only the policy's products use bf16
operands, A s + B a stays binary32.  Every rollout kernel that serves bf16 policies, against the CPU checker
with the same setting; the switch must change the results (the two settings are different arithmetic)."""
import math
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, Workload, make_inputs
from gpu_util import compare_rollout, dev, noise_to_device, probe_rollout, run_rollout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import paper_2501_15129_amd as pkg
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pkg


CASES = [
    (Workload("envf-reg-13-29-7", pop=10, envs=5, horizon=60, obs=13, hid=29, act=7, dtype=1, noise_dtype=1, seed=61, env_dtype=1), "wave_reg_bf16"),
    (Workload("envf-reg-net16-relu", pop=8, envs=2, horizon=60, obs=27, hid=16, act=8, dtype=1, noise_dtype=1, seed=62, env_dtype=1, hidden_act=1), "wave_reg_bf16"),
    (Workload("envf-lds-70-100-9", pop=4, envs=2, horizon=40, obs=70, hid=100, act=9, dtype=1, noise_dtype=1, seed=63, env_dtype=1), "wave_lds_bf16"),
    (Workload("envf-lds-depth3", pop=4, envs=2, horizon=30, obs=20, hid=40, act=5, dtype=1, noise_dtype=1, seed=64, env_dtype=1, num_hidden=3), "wave_lds_bf16"),
    (Workload("envf-mfma32", pop=6, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=65, env_dtype=1), "mfma"),
    (Workload("envf-mfma32-E3-relu", pop=4, envs=3, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=66, env_dtype=1, hidden_act=1), "mfma"),
    (Workload("envf-mfma32-E21-linear", pop=4, envs=21, horizon=30, obs=32, hid=200, act=16, dtype=1, noise_dtype=1, seed=67, env_dtype=1, out_tanh=0), "mfma"),
    (Workload("envf-mfma64", pop=4, envs=16, horizon=30, obs=60, hid=256, act=10, dtype=1, noise_dtype=1, seed=68, env_dtype=1), "mfma"),
    (Workload("envf-mfma64-obs33-fixedlen", pop=4, envs=5, horizon=50, obs=33, hid=129, act=1, dtype=1, noise_dtype=0, seed=69, env_dtype=1,
              done_thresh=math.inf), "mfma"),
]


@pytest.mark.parametrize("w,kernel", CASES, ids=lambda x: x.name if isinstance(x, Workload) else x)
def test_rollout_with_binary32_environment(es, w, kernel):
    a_mat, b_mat, theta = make_inputs(w)
    theta = (theta + np.random.default_rng(w.seed).standard_normal(theta.size) * 0.02).astype(np.float32)     # non-zero biases
    ctx = es.EsContext(w)
    assert kernel in ctx.rollout_kernel, ctx.rollout_kernel
    eps = oracle.sample_population(w, 1)
    nd = noise_to_device(ctx, eps)
    got = run_rollout(ctx, w, 1, theta, nd, a_mat, b_mat)
    ref = oracle.rollout(w, 1, theta, eps, a_mat, b_mat)
    probe = probe_rollout(w, 1, theta, eps, a_mat, b_mat, ref=ref)
    flips, worst, sens, chaotic = compare_rollout(w, got, ref, w.name, probe)
    print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens}")
    assert not chaotic
    # the same workload with a bf16 environment is different arithmetic: the GPU's two results differ
    w0 = replace(w, env_dtype=0)
    other = run_rollout(es.EsContext(w0), w0, 1, theta, nd, a_mat, b_mat)
    assert not np.array_equal(other[0], got[0])


def test_binary32_environment_with_observation_statistics(es):
    w = Workload("envf-mfma32-norm", pop=4, envs=16, horizon=40, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=70, env_dtype=1)
    a_mat, b_mat, theta = make_inputs(w)
    rng = np.random.default_rng(70)
    mean = (rng.standard_normal(w.obs) * 0.05).astype(np.float32)
    inv = (1.0 / (0.33 + rng.random(w.obs) * 0.67)).astype(np.float32)
    ctx = es.EsContext(w)
    mean_d, inv_d = dev(mean), dev(inv)
    ctx.set_obs_norm(mean_d, inv_d)
    eps = oracle.sample_population(w, 2)
    got = run_rollout(ctx, w, 2, theta, noise_to_device(ctx, eps), a_mat, b_mat)
    ref = oracle.rollout(w, 2, theta, eps, a_mat, b_mat, obs_norm=(mean, inv))
    probe = probe_rollout(w, 2, theta, eps, a_mat, b_mat, ref=ref, obs_norm=(mean, inv))
    _, _, _, chaotic = compare_rollout(w, got, ref, w.name, probe)
    assert not chaotic


def test_binary32_environment_refused_where_no_kernel_holds_it(es):
    """configs[4]'s 244 x 244 environment matrix does not fit on chip in binary32 beside the policy."""
    w = replace(CONFIGS[4], name="cfg4-envf", env_dtype=1, pop=4)
    ctx = es.EsContext(w)
    a_mat, b_mat, theta = make_inputs(w)
    with pytest.raises(es.EsError) as err:
        run_rollout(ctx, w, 0, theta, ctx.alloc_noise(), a_mat, b_mat)
    assert err.value.status == -2


def test_config3_full_size_with_binary32_environment(es):
    """configs[3] with the environment in binary32 (the reading that keeps "bf16 weights and activations" to the policy):
    whole population, contractive twin at T = 1000 held to the strict tolerance on 32 mirrored pairs, and the workload as
    specified on 32 pairs."""
    for w in (replace(CONFIGS[3].contractive(), name="cfg3-contractive-envf", env_dtype=1), replace(CONFIGS[3], name="cfg3-envf", env_dtype=1)):
        a_mat, b_mat, theta = make_inputs(w)
        ctx = es.EsContext(w)
        noise = ctx.alloc_noise()
        ctx.sample_population(0, noise)
        got = run_rollout(ctx, w, 0, theta, noise, a_mat, b_mat)
        del noise
        torch.cuda.empty_cache()
        refs, probes, subs = [], [], []
        for j in (0, 121, 300, w.pop // 2 - 8):
            eps = oracle.sample_population(w, 0, rows=(j, j + 8))
            ind = (2 * j, 2 * j + 16)
            refs.append(oracle.rollout(w, 0, theta, eps, a_mat, b_mat, individuals=ind, noise_row0=j))
            probes.append(probe_rollout(w, 0, theta, eps, a_mat, b_mat, individuals=ind, noise_row0=j, ref=refs[-1], probes=1))
            subs.append(tuple(x[ind[0]:ind[1]] for x in got))
        cat = lambda parts: tuple(np.concatenate([p[k] for p in parts]) for k in range(len(parts[0])))
        flips, worst, sens, chaotic = compare_rollout(w, cat(subs), cat(refs), w.name, cat(probes))
        print(f"[{w.name}] kernel={ctx.rollout_kernel} worst {worst:.2e} flips {flips} sensitive {sens}")
        assert not chaotic
        if "contractive" in w.name:
            assert compare_rollout.last_excused == 0 and np.all(got[1] == w.horizon)
