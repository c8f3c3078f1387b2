"""Seeded sweep over policy shapes, options and episode layouts on the two register-resident rollout kernels, horizons up
to 24 steps: every episode must meet the tolerance of its precision, except those the CPU checker's own one-ulp-nudge
probe shows to be unpinnable, which are held to bounds derived from that probe and listed."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import Workload, make_inputs
from gpu_util import compare_rollout, noise_to_device, run_rollout, probe_rollout

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def es():
    import paper_2501_15129_amd as pkg
    assert torch.cuda.is_available(), "these tests need the GPU"
    return pkg


def _sweep(es, shapes, rng, kernel, dtype_of, max_horizon):
    for n, (o, h, a, m) in enumerate(shapes):
        dt = dtype_of(rng)
        w = Workload(f"sweep{n}", pop=2 * int(rng.integers(1, 4)), envs=int(rng.integers(1, 21)), horizon=int(rng.integers(1, max_horizon + 1)),
                     obs=o, hid=h, act=a, dtype=dt, noise_dtype=dt, seed=3000 + n, hidden_act=int(rng.integers(0, 2)),
                     out_tanh=int(rng.integers(0, 2)), done_thresh=float(rng.choice([0.95, 0.5, math.inf])), num_hidden=m,
                     episodes=int(rng.integers(1, 3)))
        a_mat, b_mat, theta = make_inputs(w)
        theta = (theta + rng.standard_normal(theta.size) * 0.02).astype(np.float32)     # non-zero biases
        ctx = es.EsContext(w)
        assert kernel in ctx.rollout_kernel, (w, ctx.rollout_kernel)
        eps = oracle.sample_population(w, 1)
        got = run_rollout(ctx, w, 1, theta, noise_to_device(ctx, eps), a_mat, b_mat)
        ref = oracle.rollout(w, 1, theta, eps, a_mat, b_mat)
        probe = probe_rollout(w, 1, theta, eps, a_mat, b_mat, ref=ref)
        # episodes whose return the checker's own nudged evaluations cannot pin are held to bounds derived from that
        # spread and listed (compare_rollout prints each with its checker-side spread); everything else is strict
        flips, worst, sens, chaotic = compare_rollout(w, got, ref, f"{w.name} {o}-{h}x{m}-{a} relu{w.hidden_act} ot{w.out_tanh} T{w.horizon} E{w.envs}x{w.episodes}", probe)


def test_one_wavefront_register_kernel_shape_sweep(es):
    rng = np.random.default_rng(123)
    shapes = [(1, 1, 1, 2), (64, 64, 16, 2), (1, 64, 16, 2), (64, 1, 1, 2), (4, 16, 4, 2), (5, 17, 5, 2), (16, 33, 8, 2), (17, 32, 9, 2),
              (33, 16, 4, 2), (63, 63, 15, 2), (2, 48, 2, 2), (32, 49, 16, 2)]
    shapes += [(int(rng.integers(1, 65)), int(rng.integers(1, 65)), int(rng.integers(1, 17)), 2) for _ in range(28)]
    _sweep(es, shapes, rng, "wave_reg", lambda r: int(r.integers(0, 2)), max_horizon=24)


def test_matrix_core_kernel_shape_sweep(es):
    rng = np.random.default_rng(321)
    shapes = [(1, 128, 1, 2), (256, 256, 32, 2), (33, 129, 17, 2), (64, 256, 16, 3), (64, 255, 16, 4), (65, 200, 16, 2), (128, 130, 32, 2),
              (129, 256, 1, 2), (32, 256, 17, 2), (8, 256, 2, 3)]
    for _ in range(16):
        m = int(rng.choice([2, 2, 3, 4]))
        shapes.append((int(rng.integers(1, 65 if m > 2 else 257)), int(rng.integers(128, 257)), int(rng.integers(1, 17 if m > 2 else 33)), m))
    _sweep(es, shapes, rng, "mfma", lambda r: 1, max_horizon=24)
