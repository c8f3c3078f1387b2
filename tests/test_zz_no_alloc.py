"""es_update_static (the entry point for callers that cannot allocate) against es_update, through
the C boundary: two calls in a row on the same GPU, the second on a smaller input, each required
to reproduce es_update's outputs bit for bit (the two share their kernels and differ only in where
the binary64 partial sums live), and es_update's outputs are held to the checker's in the
stage tests.  The first call is also compared with the checker directly."""
import ctypes as C
from dataclasses import replace

import numpy as np
import pytest
import torch

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, Workload, random_fitness
from gpu_util import assert_params_close, dev

pytestmark = pytest.mark.gpu

# stored bf16 matrix of 256 MB and more: the chunked two-kernel stream whose partial rows are the scratch
BIG = replace(CONFIGS[4], name="cfg4-half", pop=2048)
# regenerated noise: the chunked reduction at any size
SMALL = Workload("regen-small", pop=64, envs=1, horizon=1, obs=17, hid=64, act=6, dtype=0, noise_dtype=2, seed=21)


def _both_ways(es, binding, w, gen, step, seed):
    """Run es_update and es_update_static from identical inputs; return the two output tuples."""
    ctx = es.EsContext(w)
    assert "grad_" in ctx.update_kernel, "this shape does not use the partial-sum scratch"
    assert ctx.workspace_bytes <= int(binding.raw_library().es_static_scratch_bytes())
    d = w.n_params
    rng = np.random.default_rng(seed)
    theta = (rng.standard_normal(d) * 0.05).astype(np.float32)
    m = (rng.standard_normal(d) * 0.01).astype(np.float32)
    v = (rng.random(d) * 1e-3).astype(np.float32)
    _, shaped = oracle.rank(random_fitness(w.pop, seed, ties=True))
    noise = ctx.alloc_noise()
    ctx.sample_population(gen, noise)
    outs = []
    for static in (False, True):
        th_d, m_d, v_d = dev(theta), dev(m), dev(v)
        g_d = torch.full((d,), float("nan"), dtype=torch.float32, device="cuda")
        if static:
            ctx.update_static(step, noise, dev(shaped), th_d, m_d, v_d, g_d)
        else:
            ws = ctx.alloc_workspace()
            ws.fill_(0xFF)
            ctx.update(step, noise, dev(shaped), th_d, m_d, v_d, g_d, ws)
        torch.cuda.synchronize()
        outs.append(tuple(t.cpu().numpy() for t in (th_d, m_d, v_d, g_d)))
    return ctx, outs, (theta, m, v, shaped)


def test_update_static_matches_update_twice_in_a_row():
    import paper_2501_15129_amd as es
    from paper_2501_15129_amd import binding
    assert torch.cuda.is_available()
    # first call: 1024 x 133120 bf16 rows (272 MB), eight chunks of partial rows (8.5 MB of scratch)
    ctx, (plain, static), (theta, m, v, shaped) = _both_ways(es, binding, BIG, gen=3, step=4, seed=5)
    for a, b, name in zip(plain, static, ("theta", "m", "v", "grad")):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"first call: {name} differs from es_update"
    eps = oracle.sample_population(BIG, 3)
    want = oracle.update(BIG, 4, eps, shaped, theta, m, v)
    for got, ref, name in zip(static, want, ("theta", "m", "v", "grad")):
        assert_params_close(got, ref, f"first call vs checker: {name}")
    del ctx, eps
    torch.cuda.empty_cache()
    # second call, smaller input, another context: the scratch still holds the first call's partial rows
    ctx2, (plain2, static2), (theta2, m2, v2, shaped2) = _both_ways(es, binding, SMALL, gen=1, step=1, seed=8)
    for a, b, name in zip(plain2, static2, ("theta", "m", "v", "grad")):
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), f"second call: {name} differs from es_update"
    want2 = oracle.update(SMALL, 1, oracle.sample_population(replace(SMALL, noise_dtype=0), 1), shaped2, theta2, m2, v2)
    for got, ref, name in zip(static2, want2, ("theta", "m", "v", "grad")):
        assert_params_close(got, ref, f"second call vs checker: {name}")


def test_update_static_refuses_what_does_not_fit():
    import paper_2501_15129_amd as es
    from paper_2501_15129_amd import binding
    lib = binding.raw_library()
    limit = int(lib.es_static_scratch_bytes())
    assert limit == 32 << 20
    # regenerated noise at a parameter count whose partial rows exceed the scratch
    w = replace(CONFIGS[4], name="too-wide", noise_dtype=3, obs=2048, hid=2048, act=64, pop=64)
    ctx = es.EsContext(w)
    assert ctx.workspace_bytes > limit
    one = torch.zeros(1, device="cuda")
    rc = lib.es_update_static(ctx._h, 1, None, one.data_ptr(), one.data_ptr(), one.data_ptr(), one.data_ptr(), None, None)
    assert rc == binding.ES_EUNSUPPORTED
    assert b"built-in scratch" in lib.es_last_error(ctx._h)
