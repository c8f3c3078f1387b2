"""Pins for the integer and bit-defined parts of the CPU checker: Philox words, the
Gaussian transform, bf16 rounding, the perturbation and the environment reset.

Each pin compares the checker with something other than itself: published
known-answer vectors, a binary64 libm evaluation of the mathematical definition,
sample statistics of the normal law, or a library's rounding.
"""
import math
from dataclasses import replace

import numpy as np
import pytest
import scipy.stats
import torch

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, Workload

TINY = Workload("tiny", pop=8, envs=2, horizon=5, obs=3, hid=4, act=2, dtype=0, noise_dtype=0, seed=11)


def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in (golden_dir / "philox4x32_10_kat.txt").read_text().splitlines()
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        assert oracle.philox4x32_10(v[0:4], v[4:6]) == v[6:10]


def test_philox_counter_and_key_sensitivity():
    # distinct counters / keys give distinct blocks (bijection in the counter for a fixed key)
    seen = set()
    for c0 in range(64):
        for c1 in range(4):
            for k0 in range(2):
                seen.add(tuple(oracle.philox4x32_10((c0, c1, 0, 1), (k0, 0))))
    assert len(seen) == 64 * 4 * 2


def _box_muller_f64(xa, xb):
    k1 = (np.asarray(xa, dtype=np.uint64) >> 8) + 1
    k2 = np.asarray(xb, dtype=np.uint64) >> 8
    u1 = k1.astype(np.float64) / 2.0 ** 24
    ang = 2.0 * np.pi * k2.astype(np.float64) / 2.0 ** 24
    rad = np.sqrt(-2.0 * np.log(u1))
    return rad * np.cos(ang), rad * np.sin(ang)


def test_gauss_pair_matches_box_muller_definition():
    rng = np.random.default_rng(5)
    xa = rng.integers(0, 2 ** 32, size=100_000, dtype=np.uint64)
    xb = rng.integers(0, 2 ** 32, size=100_000, dtype=np.uint64)
    # edge words: smallest / largest radius, every octant boundary and both sides of it
    edges = [0, 0xFF, 0x100, 0xFFFFFFFF, 0xFFFFFF00, 0x7FFFFFFF, 0x80000000, 0xB504F300, 0xB504F400]
    for o in range(8):
        edges += [o << 29, (o << 29) + 0x100, ((o + 1) << 29) - 0x100 & 0xFFFFFFFF]
    ea, eb = np.meshgrid(np.array(edges, dtype=np.uint64), np.array(edges, dtype=np.uint64))
    xa = np.concatenate([xa, ea.ravel()])
    xb = np.concatenate([xb, eb.ravel()])
    zc, zs = _box_muller_f64(xa, xb)
    got = np.array([oracle.gauss_pair(int(a), int(b)) for a, b in zip(xa, xb)], dtype=np.float64)
    assert np.max(np.abs(got[:, 0] - zc)) < 1e-6
    assert np.max(np.abs(got[:, 1] - zs)) < 1e-6
    assert np.max(np.abs(got)) < 5.78          # sqrt(2 * 24 ln 2)
    # largest uniform (k1 = 2^24) has radius exactly zero
    assert oracle.gauss_pair(0xFFFFFFFF, 12345) == (0.0, 0.0)


def test_noise_is_standard_normal():
    w = replace(TINY, pop=64, obs=60, hid=100, act=10)      # D = 17 210, 32 rows -> 550 720 samples
    eps = oracle.sample_population(w, gen=3).astype(np.float64).ravel()
    n = eps.size
    assert abs(eps.mean()) < 4.0 / math.sqrt(n)
    assert abs(eps.var() - 1.0) < 4.0 * math.sqrt(2.0 / n)
    assert abs(scipy.stats.skew(eps)) < 4.0 * math.sqrt(6.0 / n)
    assert abs(scipy.stats.kurtosis(eps)) < 4.0 * math.sqrt(24.0 / n)
    assert scipy.stats.kstest(eps, "norm").pvalue > 1e-3
    # rows, columns and generations are distinct streams
    m = eps.reshape(32, -1)
    assert abs(np.corrcoef(m[0], m[1])[0, 1]) < 5.0 / math.sqrt(m.shape[1])
    eps_g4 = oracle.sample_population(w, gen=4).astype(np.float64).ravel()
    assert abs(np.corrcoef(eps, eps_g4)[0, 1]) < 5.0 / math.sqrt(n)
    other_seed = oracle.sample_population(replace(w, seed=12), gen=3).astype(np.float64).ravel()
    assert abs(np.corrcoef(eps, other_seed)[0, 1]) < 5.0 / math.sqrt(n)


def test_noise_stream_layout():
    # element d of row j is variate d%4 of block (d//4, j, gen, stream 1) keyed by the seed
    w = replace(TINY, seed=(7 << 32) | 9)
    gen = 6
    eps = oracle.sample_population(w, gen)
    d_count = w.n_params
    assert eps.shape == (w.pop // 2, d_count)
    for j in (0, 3):
        for d in (0, 1, 2, 3, 4, 7, d_count - 1):
            words = oracle.philox4x32_10((d // 4, j, gen, 1), (9, 7))
            q = d % 4
            z = oracle.gauss_pair(words[q & 2], words[(q & 2) + 1])[q & 1]
            assert eps[j, d] == np.float32(z)
    # row subset call agrees with the full call
    assert np.array_equal(oracle.sample_population(w, gen, rows=(1, 3)), eps[1:3])


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.001953125, 1.005859375, -2.5e-3, 3.0e38],
                                 dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(oracle.bf16_round(x).view(np.uint32), want.view(np.uint32))
    w = replace(TINY, noise_dtype=1)
    e32 = oracle.sample_population(TINY, 0)
    e16 = oracle.sample_population(w, 0)
    want = torch.from_numpy(e32).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(e16, want)


def test_perturbation():
    w = TINY
    rng = np.random.default_rng(1)
    theta = rng.standard_normal(w.n_params).astype(np.float32)
    eps = oracle.sample_population(w, 0)
    for i in range(w.pop):
        got = oracle.perturb(w, theta, eps, i)
        sign = -1.0 if i % 2 else 1.0
        sig = float(np.float32(w.sigma))
        # product of two binary32 numbers is exact in binary64; one more rounding to binary32
        want = (sign * sig * eps[i // 2].astype(np.float64) + theta.astype(np.float64))
        assert np.max(np.abs(got - want)) <= np.max(np.abs(want)) * 2.0 ** -23
        assert np.mean(got == want.astype(np.float32)) > 0.99
    # mirrored pair is symmetric about theta; sigma = 0 reproduces theta bit for bit
    p0, p1 = oracle.perturb(w, theta, eps, 2), oracle.perturb(w, theta, eps, 3)
    assert np.allclose(p0.astype(np.float64) + p1, 2.0 * theta.astype(np.float64), atol=2e-7)
    w0 = replace(w, sigma=0.0)
    for i in range(w.pop):
        assert np.array_equal(oracle.perturb(w0, theta, eps, i).view(np.uint32), theta.view(np.uint32))
    # without mirroring every individual has its own row and sign +1
    wn = replace(w, antithetic=0)
    eps_n = oracle.sample_population(wn, 0)
    assert eps_n.shape[0] == w.pop and np.array_equal(eps_n[: w.pop // 2], eps)
    got = oracle.perturb(wn, theta, eps_n, 5)
    want = (float(np.float32(w.sigma)) * eps_n[5].astype(np.float64) + theta).astype(np.float32)
    assert np.mean(got == want) > 0.99
    # bf16 mode rounds the perturbed parameters
    wb = replace(w, dtype=1)
    gb = oracle.perturb(wb, theta, eps, 1)
    want = torch.from_numpy(oracle.perturb(w, theta, eps, 1)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(gb, want)


def test_reset_is_uniform_and_keyed():
    w = replace(TINY, obs=64)
    s = np.stack([oracle.reset(w, gen=0, e=e) for e in range(200)]).astype(np.float64)
    assert s.min() >= -0.1 and s.max() < 0.1
    n = s.size
    assert abs(s.mean()) < 4 * (0.2 / math.sqrt(12)) / math.sqrt(n)
    assert abs(s.var() - 0.2 ** 2 / 12) < 5 * (0.2 ** 2) * math.sqrt(1 / 180.0) / math.sqrt(n)
    assert scipy.stats.kstest((s.ravel() + 0.1) / 0.2, "uniform").pvalue > 1e-3
    assert not np.array_equal(oracle.reset(w, 0, 0), oracle.reset(w, 1, 0))
    assert not np.array_equal(oracle.reset(w, 0, 0), oracle.reset(w, 0, 1))
    # layout: word k%4 of block (k//4, e, gen, stream 2), top 24 bits, affine map
    words = oracle.philox4x32_10((5 // 4, 7, 2, 2), (w.seed & 0xFFFFFFFF, w.seed >> 32))
    u = (words[5 % 4] >> 8) / 2.0 ** 24
    assert abs(float(oracle.reset(w, 2, 7)[5]) - (0.2 * u - 0.1)) < 1e-8


def test_param_count_matches_shapes():
    for w, d in zip(CONFIGS, (1539, 5702, 5702, 75016, 132881)):
        assert oracle.param_count(w) == d == w.n_params


# ---- pre-built shared noise table (paper Sec. 5.1: the noise-table variant, after Salimans et al. 2017) ----
def test_table_entries_are_the_pinned_generator_and_transform_on_stream_three():
    import torch
    w = CONFIGS[1]
    key = [w.seed & 0xFFFFFFFF, w.seed >> 32]
    t0, t1 = 1000, 1064
    tab = oracle.table_slice(w, t0, t1, False)
    for t in range(t0, t1):
        words = oracle.philox4x32_10([t // 4, 0, 0, 3], key)
        za, zb = oracle.gauss_pair(words[2 * ((t % 4) // 2)], words[2 * ((t % 4) // 2) + 1])
        want = np.float32(zb if t % 2 else za)
        assert tab[t - t0].view(np.uint32) == want.view(np.uint32)
    rounded = oracle.table_slice(w, t0, t1, True)
    lib = torch.from_numpy(tab).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(rounded.view(np.uint32), lib.view(np.uint32))
    # slices agree with one another and differ from the per-generation noise stream
    assert np.array_equal(oracle.table_slice(w, 0, 2048, False)[t0:t1], tab)
    assert not np.array_equal(oracle.sample_population(w, 0, rows=(0, 1))[0, :64], oracle.table_slice(w, 0, 64, False))


def test_table_moments():
    tab = oracle.table_slice(CONFIGS[0], 0, 1 << 18, False).astype(np.float64)
    n = tab.size
    assert abs(tab.mean()) < 5 / np.sqrt(n) and abs(tab.var() - 1) < 5 * np.sqrt(2 / n)
    assert abs(np.mean(tab ** 3)) < 5 * np.sqrt(15 / n) and abs(np.mean(tab ** 4) - 3) < 5 * np.sqrt(96 / n)
    assert abs(np.corrcoef(tab[:-1], tab[1:])[0, 1]) < 5 / np.sqrt(n)


def test_table_offsets_are_aligned_in_range_and_follow_their_counter():
    w = CONFIGS[3]
    key = [w.seed & 0xFFFFFFFF, w.seed >> 32]
    length, span = 1 << 22, 75264
    offs = oracle.table_offsets(w, 5, length, span)
    assert offs.size == w.noise_rows and np.all(offs % 8 == 0) and np.all(offs.astype(np.int64) + span <= length)
    m = (length - span) // 8 + 1
    for j in (0, 1, 17, w.noise_rows - 1):
        assert int(offs[j]) == 8 * (oracle.philox4x32_10([j, 5, 0, 4], key)[0] % m)
    assert not np.array_equal(offs, oracle.table_offsets(w, 6, length, span))
    # spread over the table: the offsets of 512 rows fall into all eight eighths of the range
    assert len(set((offs.astype(np.int64) * 8 // (length - span + 8)).tolist())) == 8
    # the smallest admissible table has a single place for a row
    assert np.all(oracle.table_offsets(w, 5, span, span) == 0)


def test_table_rows_are_slices_of_the_table():
    w = CONFIGS[0]
    length = 8192
    tab = oracle.table_slice(w, 0, length, False)
    offs = oracle.table_offsets(w, 2, length, 2048)
    rows = oracle.table_rows(w, 2, length, 2048, False)
    assert rows.shape == (w.noise_rows, w.n_params)
    for j in range(w.noise_rows):
        assert np.array_equal(rows[j], tab[offs[j]:offs[j] + w.n_params])
