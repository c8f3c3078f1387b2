"""Pins for the CPU checker's ranking, gradient estimate and Adam step."""
from dataclasses import replace

import numpy as np
import scipy.stats
import torch

import oracle
from paper_2501_15129_amd.workloads import Workload, random_fitness

W = Workload("tiny", pop=10, envs=1, horizon=1, obs=3, hid=4, act=2, dtype=0, noise_dtype=0, seed=31)


def test_rank_against_stable_sort_and_invariants():
    for n, ties in ((2, False), (7, False), (64, True), (1000, True)):
        f = random_fitness(n, seed=n, ties=ties)
        r, u = oracle.rank(f)
        order = np.argsort(f, kind="stable")
        want = np.empty(n, dtype=np.int32)
        want[order] = np.arange(n, dtype=np.int32)
        assert np.array_equal(r, want)
        assert sorted(r.tolist()) == list(range(n))
        assert np.array_equal(u, (r.astype(np.float32) / np.float32(n - 1)) - np.float32(0.5))
        assert abs(float(u.astype(np.float64).sum())) < 1e-4
        if not ties:
            assert np.array_equal(r, scipy.stats.rankdata(f, method="ordinal").astype(np.int32) - 1)
        # invariant under a strictly increasing map of the fitness
        r2, _ = oracle.rank(np.arctan(f.astype(np.float64) / 50.0).astype(np.float32) if not ties else f * 2 + 1)
        assert np.array_equal(r, r2)


def test_rank_degenerate_inputs():
    r, u = oracle.rank(np.full(9, 3.25, dtype=np.float32))
    assert np.array_equal(r, np.arange(9)) and u[0] == -0.5 and u[-1] == 0.5
    r, _ = oracle.rank(np.array([0.0, -0.0, 0.0, -1.0], dtype=np.float32))     # -0 ties with +0
    assert r.tolist() == [1, 2, 3, 0]
    f = np.array([1.0, np.inf, -np.inf, np.nan, 0.5], dtype=np.float32)        # no error; NaN sorts last
    r, u = oracle.rank(f)
    assert r.tolist() == [2, 3, 0, 4, 1] and np.all(np.isfinite(u))
    r, u = oracle.rank(np.array([5.0], dtype=np.float32))
    assert r.tolist() == [0] and u.tolist() == [0.0]


def _grad_only(w, noise, shaped):
    d = w.n_params
    z = np.zeros(d, dtype=np.float32)
    return oracle.update(replace(w, weight_decay=0.0), 1, noise, shaped, z, z, z)[3].astype(np.float64)


def test_gradient_estimate_closed_form_on_quadratic():
    """With the raw quadratic fitness f(x) = -|x - c|^2 / 2 used as the weights and mirrored
    pairs theta +- sigma eps_j, the estimate equals -(2/N) sum_j eps_j eps_j^T (theta - c)
    exactly, for any sigma."""
    rng = np.random.default_rng(3)
    d = W.n_params
    eps = oracle.sample_population(W, 0).astype(np.float64)
    theta = rng.standard_normal(d) * 0.05
    c = theta + rng.standard_normal(d) * 0.05
    sig = float(np.float32(W.sigma))
    fit = np.empty(W.pop)
    for j in range(W.pop // 2):
        fit[2 * j] = -0.5 * np.sum((theta + sig * eps[j] - c) ** 2)
        fit[2 * j + 1] = -0.5 * np.sum((theta - sig * eps[j] - c) ** 2)
    got = _grad_only(W, eps.astype(np.float32), fit.astype(np.float32))
    want = -(2.0 / W.pop) * (eps.T @ (eps @ (theta - c)))
    # the weights are passed in binary32: their rounding (|f| 2^-24) divided by N sigma bounds the error
    tol = np.max(np.abs(fit)) * 2.0 ** -23 / sig * np.max(np.abs(eps)) + 1e-6 * np.max(np.abs(want))
    assert np.max(np.abs(got - want)) < tol
    assert tol < 0.02 * np.max(np.abs(want))
    # unmirrored sampling: g = 1/(N sigma) sum_i w_i eps_i, a plain matrix-vector product
    wn = replace(W, antithetic=0)
    eps_n = oracle.sample_population(wn, 0)
    wts = rng.standard_normal(W.pop).astype(np.float32)
    got = _grad_only(wn, eps_n, wts)
    want = eps_n.astype(np.float64).T @ wts.astype(np.float64) / (W.pop * sig)
    assert np.allclose(got, want, rtol=1e-6, atol=1e-7)


def test_gradient_estimate_two_individuals_enumerated():
    w = replace(W, pop=2)
    eps = oracle.sample_population(w, 0)
    sig = float(np.float32(w.sigma))
    for fit, sign in (([1.0, 2.0], -1.0), ([2.0, 1.0], 1.0), ([1.0, 1.0], -1.0)):   # tie -> index order
        _, u = oracle.rank(np.array(fit, dtype=np.float32))
        got = _grad_only(w, eps, u)
        assert np.allclose(got, sign * eps[0].astype(np.float64) / (2.0 * sig), rtol=1e-6)


def _drive(w, grads_hat, theta0, steps):
    """Feed a chosen search gradient through the checker: N = 2 mirrored, weights (+1/2, -1/2) and
    noise row = g * 2 sigma, so that the estimate equals g up to binary32 rounding of the row."""
    w2 = replace(w, pop=2)
    sig = float(np.float32(w2.sigma))
    th, m, v = theta0.astype(np.float32), np.zeros_like(theta0, dtype=np.float32), np.zeros_like(theta0, dtype=np.float32)
    out, used = [], []
    for k in range(steps):
        row = (grads_hat[k] * 2.0 * sig).astype(np.float32)[None, :]
        th, m, v, g = oracle.update(w2, k + 1, row, np.array([0.5, -0.5], dtype=np.float32), th, m, v)
        used.append(row[0].astype(np.float64) / (2.0 * sig))
        out.append((th.copy(), m.copy(), v.copy(), g.copy()))
    return out, used


def test_adam_against_library_optimizer():
    rng = np.random.default_rng(8)
    d = W.n_params
    theta0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    for wd in (0.0, 0.005):
        w = replace(W, weight_decay=wd)
        ghat = [rng.standard_normal(d) * (0.3 if k % 2 else 3.0) for k in range(6)]
        out, used = _drive(w, ghat, theta0, steps=6)
        p = torch.tensor(theta0.astype(np.float64), requires_grad=True)
        opt = torch.optim.Adam([p], lr=float(np.float32(w.lr)),
                               betas=(float(np.float32(w.beta1)), float(np.float32(w.beta2))),
                               eps=float(np.float32(w.adam_eps)), weight_decay=float(np.float32(wd)))
        for k in range(6):
            opt.zero_grad()
            p.grad = torch.from_numpy(-used[k])          # ascent on fitness = descent on its negative
            opt.step()
            # the checker stores theta, m, v in binary32 between steps: compare with that granularity
            assert np.allclose(out[k][0], p.detach().numpy(), rtol=0, atol=3e-7 * (k + 1))
            assert np.allclose(out[k][3], used[k], rtol=1e-6, atol=1e-9)
            st = opt.state[p]
            assert np.allclose(out[k][1], st["exp_avg"].numpy(), rtol=1e-5, atol=1e-7)
            assert np.allclose(out[k][2], st["exp_avg_sq"].numpy(), rtol=1e-5, atol=1e-9)


def test_adam_closed_forms():
    rng = np.random.default_rng(9)
    d = W.n_params
    w = replace(W, weight_decay=0.0)
    theta0 = (rng.standard_normal(d) * 0.1).astype(np.float32)
    g = rng.standard_normal(d)
    out, used = _drive(w, [g] * 4, theta0, steps=4)
    lr, eps_a = float(np.float32(w.lr)), float(np.float32(w.adam_eps))
    grad = -used[0]
    # first step from m = v = 0, and every later step under a constant gradient, moves by
    # -lr * grad / (|grad| + eps)
    prev = theta0.astype(np.float64)
    for k in range(4):
        step = out[k][0].astype(np.float64) - prev
        assert np.allclose(step, -lr * grad / (np.abs(grad) + eps_a), rtol=1e-4, atol=2e-7)
        prev = out[k][0].astype(np.float64)
    # weight decay only: zero search gradient, grad = lambda * theta
    w = replace(W, weight_decay=0.005)
    out, _ = _drive(w, [np.zeros(d)], theta0, steps=1)
    gr = float(np.float32(0.005)) * theta0.astype(np.float64)
    assert np.allclose(out[0][0], theta0 - lr * gr / (np.abs(gr) + eps_a), rtol=0, atol=2e-7)
    assert np.allclose(out[0][1], (1 - float(np.float32(w.beta1))) * gr, rtol=1e-5, atol=1e-12)
