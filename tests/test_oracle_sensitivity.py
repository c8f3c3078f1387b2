"""The sensitivity probe (one-ulp operand nudges, evaluated by the CPU checker alone) and the two
regimes it tells apart: the contractive twins of the benchmark workloads damp a nudge far below the
tolerance at the full horizon, the original configs[4] under the fixed-length protocol amplifies it."""
from dataclasses import replace

import numpy as np
import pytest

import oracle
from paper_2501_15129_amd.workloads import CONFIGS, make_inputs
from sensitivity import nudged_inputs, probe_rollout, spread_of

RET_RTOL = {0: 1e-4, 1: 2e-2}


def _spread(w, pair, gen=0, probes=2):
    a_mat, b_mat, theta = make_inputs(w)
    eps = oracle.sample_population(w, gen, rows=(pair, pair + 1))
    ind = (2 * pair, 2 * pair + 2)
    ref = oracle.rollout(w, gen, theta, eps, a_mat, b_mat, individuals=ind, noise_row0=pair)
    probe = probe_rollout(w, gen, theta, eps, a_mat, b_mat, ref=ref, individuals=ind, noise_row0=pair, probes=probes)
    return ref, spread_of(probe, ref[0], ref[1])


def test_nudges_move_a_handful_of_operands_by_one_ulp():
    for w in (CONFIGS[1], CONFIGS[3]):
        a_mat, b_mat, theta = make_inputs(w)
        th, a_n, b_n = nudged_inputs(w, theta, a_mat, b_mat, seed=5)
        moved = np.flatnonzero(th != theta)
        assert 0 < moved.size <= 8 * 3
        rel = np.abs(th[moved].astype(np.float64) - theta[moved]) / np.abs(theta[moved])
        lo, hi = (2.0 ** -9, 2.0 ** -7) if w.dtype == 1 else (2.0 ** -25, 2.0 ** -23)
        assert np.all((rel >= lo * 0.999) & (rel <= hi * 1.001))
        base_a = oracle.bf16_round(a_mat) if w.dtype == 1 else a_mat
        assert 0 < np.count_nonzero(a_n != base_a) <= 8 and 0 < np.count_nonzero(b_n != (oracle.bf16_round(b_mat) if w.dtype == 1 else b_mat)) <= 8
        if w.dtype == 1:        # nudged environment entries are still bf16 values
            assert np.array_equal(oracle.bf16_round(a_n), a_n)


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_contractive_twins_damp_a_nudge_at_full_horizon(idx):
    """Same shapes, T = 1000, fixed length: no return moves by more than 1/8 of the tolerance."""
    w = CONFIGS[idx].contractive()
    assert (w.pop, w.envs, w.horizon, w.obs, w.hid, w.act, w.dtype) == tuple(
        getattr(CONFIGS[idx], k) for k in ("pop", "envs", "horizon", "obs", "hid", "act", "dtype"))
    ref, (spread, mean_spread, _) = _spread(w, pair=w.pop // 4, probes=1 if idx >= 3 else 2)
    assert np.all(ref[1] == w.horizon)
    assert float(spread.max()) <= 0.125 * RET_RTOL[w.dtype], float(spread.max())
    # the twin is not a trivial workload: the loop settles away from the origin, and mirrored individuals differ
    per_step = ref[0] / w.horizon
    assert np.all(per_step < 0.98) and np.all(per_step > 0.3)
    assert abs(float(ref[2][0]) - float(ref[2][1])) > 1e-3 * abs(float(ref[2][0])) * (0.02 if idx < 3 else 0.0)


def test_original_cfg4_fixed_length_amplifies_a_nudge():
    """The probe sees what a binary32 re-evaluation with the roundings in the same places cannot:
    after 60 steps one bf16 ulp on a few operands has moved returns by more than the tolerance allows."""
    w = replace(CONFIGS[4].fixed_length(), horizon=60)
    ref, (spread, _, _) = _spread(w, pair=0, probes=2)
    assert float(spread.max()) > 0.125 * RET_RTOL[1]
