"""Pins for the checker's ARS and VanillaES steps (paper Sec. 4, App. B Tables 5(a) and 5(c);
algorithms as published by Mania et al. 2018 and Chrabaszcz et al. 2018).  Each test ties the
checker to something other than itself: a hand-worked example, an invariance the mathematics
fixes, a matrix closed form evaluated with a library product, or a direct evaluation of the
published formula written a different way (sort-based, in numpy binary64)."""
import math
from dataclasses import replace

import numpy as np
import pytest

import oracle
from paper_2501_15129_amd.workloads import Workload

W = Workload("sib", pop=12, envs=1, horizon=1, obs=3, hid=4, act=2, dtype=0, noise_dtype=0, seed=3, lr=0.02, sigma=0.03)
D = W.n_params


def _rng_case(seed, pop, ties=False):
    rng = np.random.default_rng(seed)
    f = rng.standard_normal(pop).astype(np.float32) * 3 + 1
    if ties:
        f[rng.integers(0, pop, size=pop // 3)] = f[0]
    return rng, f


# ------------------------------------------------------------------ ARS
def test_ars_hand_worked_example():
    # two directions e_x, e_y; returns (3, 1) and (10, 4); keep the best one (b = 1):
    # direction 1 is kept, sigma_R = std{10, 4} = 3, step = lr / (1 * 3) * (10 - 4) * e_y = 2 lr e_y
    w = replace(W, pop=4, obs=1, hid=1, act=1)          # D = 2 + 2 + 2 = 6; use the first two coordinates
    d = w.n_params
    noise = np.zeros((2, d), dtype=np.float32)
    noise[0, 0], noise[1, 1] = 1.0, 1.0
    f = np.array([3, 1, 10, 4], dtype=np.float32)
    rank, shaped = oracle.rank_ars(f, 1)
    assert rank.tolist() == [1, 1, 0, 0]
    assert np.allclose(shaped, [0, 0, 10 / 3, 4 / 3], rtol=1e-6)
    theta, g = oracle.update_ars(w, 1, noise, shaped, np.zeros(d, dtype=np.float32))
    want = np.zeros(d)
    want[1] = 2 * 0.02
    assert np.allclose(theta, want, rtol=1e-6, atol=1e-9)
    assert np.allclose(g[1], 2.0, rtol=1e-6) and np.all(g[[0, 2, 3, 4, 5]] == 0)


@pytest.mark.parametrize("seed,b,ties", [(0, 1, False), (1, 3, False), (2, 6, False), (3, 4, True), (4, 2, True)])
def test_ars_matches_published_formula_written_with_sorts(seed, b, ties):
    rng, f = _rng_case(seed, W.pop, ties)
    noise = rng.standard_normal((W.pop // 2, D)).astype(np.float32)
    theta = rng.standard_normal(D).astype(np.float32) * 0.1
    rank, shaped = oracle.rank_ars(f, b)
    got, _ = oracle.update_ars(W, b, noise, shaped, theta)
    fp, fm = f[0::2].astype(np.float64), f[1::2].astype(np.float64)
    order = sorted(range(W.pop // 2), key=lambda j: (-max(fp[j], fm[j]), j))
    kept = order[:b]
    assert [int(rank[2 * j]) for j in order] == list(range(W.pop // 2))
    sigma_r = np.std(np.concatenate([fp[kept], fm[kept]]))
    step = sum((fp[j] - fm[j]) * noise[j].astype(np.float64) for j in kept)
    want = theta.astype(np.float64) + 0.02 / (b * sigma_r) * step
    assert np.allclose(got, want, rtol=2e-6, atol=1e-8)


def test_ars_invariant_under_positive_scaling_and_shift_of_returns():
    rng, f = _rng_case(7, W.pop)
    noise = rng.standard_normal((W.pop // 2, D)).astype(np.float32)
    theta = rng.standard_normal(D).astype(np.float32) * 0.1
    base, _ = oracle.update_ars(W, 3, noise, oracle.rank_ars(f, 3)[1], theta)
    for g in (f * 4.0, f * 0.3, f + 2.0, f * 8.0 - 16.0):
        other, _ = oracle.update_ars(W, 3, noise, oracle.rank_ars(g.astype(np.float32), 3)[1], theta)
        assert np.allclose(other, base, rtol=1e-4, atol=1e-7)           # binary32 returns: shift/scale round them


def test_ars_linear_fitness_all_directions_closed_form():
    # F(theta') = c . theta'  =>  F+ - F- = 2 sigma c . delta_j ; with every direction kept the step is
    # lr * 2 sigma / (R sigma_R) * Delta^T Delta c, a matrix expression evaluated by the library product
    rng = np.random.default_rng(11)
    r = W.pop // 2
    delta = rng.standard_normal((r, D)).astype(np.float32)
    c = rng.standard_normal(D)
    theta = rng.standard_normal(D).astype(np.float32) * 0.1
    sigma = 0.03
    f = np.empty(W.pop, dtype=np.float64)
    f[0::2] = (theta + sigma * delta.astype(np.float64)) @ c
    f[1::2] = (theta - sigma * delta.astype(np.float64)) @ c
    f32 = f.astype(np.float32)
    got, _ = oracle.update_ars(W, r, delta, oracle.rank_ars(f32, r)[1], theta)
    f64 = f32.astype(np.float64)
    dd = delta.astype(np.float64)
    want = theta + 0.02 / (r * np.std(f64)) * (dd.T @ (f64[0::2] - f64[1::2]))
    assert np.allclose(got, want, rtol=2e-6, atol=1e-8)
    # and against the analytic right-hand side (returns rounded to binary32 cost ~1e-6 relative)
    analytic = theta + 0.02 * 2 * sigma / (r * np.std(f)) * (dd.T @ (dd @ c))
    assert np.allclose(got, analytic, rtol=1e-3, atol=1e-6)


def test_ars_degenerate_equal_returns_leave_theta_unchanged():
    noise = np.ones((W.pop // 2, D), dtype=np.float32)
    theta = np.full(D, 0.25, dtype=np.float32)
    rank, shaped = oracle.rank_ars(np.full(W.pop, 1.5, dtype=np.float32), 2)
    assert rank.tolist() == [j // 2 for j in range(W.pop)] and np.all(shaped == 0)
    got, _ = oracle.update_ars(W, 2, noise, shaped, theta)
    assert np.array_equal(got, theta)


# ------------------------------------------------------------------ VanillaES
WV = replace(W, antithetic=0, sigma=0.02)


@pytest.mark.parametrize("mu", [1, 2, 5, 12])
def test_vanilla_weights_are_the_published_log_rank_weights(mu):
    _, f = _rng_case(mu, WV.pop, ties=(mu == 5))
    rank, shaped = oracle.rank_vanilla(f, mu)
    order = sorted(range(WV.pop), key=lambda i: (-f[i], i))
    assert [int(rank[i]) for i in order] == list(range(WV.pop))
    w = np.log(mu + 0.5) - np.log(np.arange(1, mu + 1))
    w /= w.sum()
    assert np.allclose(shaped[order[:mu]], w, rtol=1e-6)
    assert np.all(shaped[order[mu:]] == 0)
    assert abs(float(shaped.astype(np.float64).sum()) - 1.0) < 1e-6
    assert np.all(np.diff(shaped[order[:mu]]) < 0) or mu == 1


def test_vanilla_hand_worked_weights():
    # mu = 2: (ln 2.5 - ln 1, ln 2.5 - ln 2) / sum = (0.9162907, 0.2231436) / 1.1394343 = (0.804163, 0.195837)
    _, shaped = oracle.rank_vanilla(np.array([0.0, 5.0, 1.0], dtype=np.float32), 2)
    assert np.allclose(shaped, [0.0, 0.804163, 0.195837], atol=2e-6)


def test_vanilla_mu_one_returns_the_best_offspring():
    rng, f = _rng_case(5, WV.pop)
    noise = rng.standard_normal((WV.pop, D)).astype(np.float32)
    theta = rng.standard_normal(D).astype(np.float32) * 0.1
    got, _ = oracle.update_vanilla(WV, noise, oracle.rank_vanilla(f, 1)[1], theta)
    best = int(np.argmax(f))
    assert np.allclose(got, oracle.perturb(WV, theta, noise, best), rtol=2e-7, atol=1e-9)


@pytest.mark.parametrize("seed,mu", [(0, 3), (1, 6), (2, 12)])
def test_vanilla_recombination_matches_weighted_mean_of_selected_offspring(seed, mu):
    rng, f = _rng_case(seed, WV.pop, ties=(seed == 1))
    noise = rng.standard_normal((WV.pop, D)).astype(np.float32)
    theta = rng.standard_normal(D).astype(np.float32) * 0.1
    got, g = oracle.update_vanilla(WV, noise, oracle.rank_vanilla(f, mu)[1], theta)
    order = sorted(range(WV.pop), key=lambda i: (-f[i], i))[:mu]
    w = np.array([math.log(mu + 0.5) - math.log(k) for k in range(1, mu + 1)])
    w /= w.sum()
    offspring = theta.astype(np.float64) + np.float64(np.float32(0.02)) * noise[order].astype(np.float64)
    want = (w[:, None] * offspring).sum(axis=0)
    assert np.allclose(got, want, rtol=2e-6, atol=1e-8)
    assert np.allclose(g, want - theta, rtol=1e-4, atol=1e-7)
