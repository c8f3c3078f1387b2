"""How sensitive is an episode's return to the last bit of its operands?  Measured on the CPU
checker ALONE: the same episodes are evaluated again (binary64, like the reference) after a handful
of operands - weights of every layer, entries of the environment matrices - have been moved by one
unit in the last place of the operand type (binary32, or bf16 when the workload rounds its operands).
A closed loop that amplifies such a nudge cannot be tracked by ANY finite-precision evaluation, the
kernels' included; one that damps it can be held to the strict tolerance at any horizon.

Unlike a second evaluation in narrower arithmetic with the roundings at the same places, this sees
chaos in bf16 mode too: there both evaluations round at the same points, agree step for step for a long
time, and hide the amplification that a single different rounding decision would meet.
"""
from __future__ import annotations

import numpy as np

import oracle

NUDGED_PER_BLOCK = 8      # operands moved in each of: every weight matrix, A, B
PROBES = 3                # independent nudge sets; the spread is the largest deviation over them


def _ulp_step(x: np.ndarray, bf16: bool, sign: np.ndarray) -> np.ndarray:
    """x moved by one unit in the last place of its operand type, in direction `sign` (+1 / -1)."""
    x = np.asarray(x, dtype=np.float32)
    if not bf16:
        return np.nextafter(x, np.where(sign > 0, np.inf, -np.inf).astype(np.float32)).astype(np.float32)
    # bf16 has 8 significant bits: one ulp of x is 2^(exponent(x) - 7); zero moves to the smallest normal step used here
    mag = np.maximum(np.abs(x).astype(np.float64), 2.0 ** -100)
    ulp = 2.0 ** (np.floor(np.log2(mag)) - 7.0)
    return (x.astype(np.float64) + sign * ulp).astype(np.float32)


def nudged_inputs(w, theta, a_mat, b_mat, seed: int):
    """Copies of (theta, A, B) with NUDGED_PER_BLOCK entries of every weight matrix, of A and of B moved by one ulp."""
    from paper_2501_15129_amd.workloads import layer_shapes
    rng = np.random.default_rng([int(seed), 0x4E554447])
    bf16 = w.dtype == 1
    theta = np.array(theta, dtype=np.float32, copy=True)
    off = 0
    for shp in layer_shapes(w):
        n = int(np.prod(shp))
        if len(shp) == 2:
            idx = off + rng.choice(n, size=min(NUDGED_PER_BLOCK, n), replace=False)
            theta[idx] = _ulp_step(theta[idx], bf16, rng.choice([-1.0, 1.0], size=idx.size))
        off += n
    out = [theta]
    for mat in (a_mat, b_mat):
        m = np.array(mat, dtype=np.float32, copy=True)
        if bf16:                                    # the operand is the bf16-rounded entry: step from there
            m = oracle.bf16_round(m)
        flat = m.ravel()
        idx = rng.choice(flat.size, size=min(NUDGED_PER_BLOCK, flat.size), replace=False)
        flat[idx] = _ulp_step(flat[idx], bf16, rng.choice([-1.0, 1.0], size=idx.size))
        out.append(m)
    return tuple(out)


def probe_rollout(w, gen, theta, eps, a_mat, b_mat, ref, individuals=None, noise_row0=0, obs_norm=None, probes=None):
    """The checker's returns of the same episodes under one-ulp operand nudges: (returns [n, E, P] f64,
    ep_len [n, E, P] i32) for P nudge sets.  `ref` is unused but names the evaluation the probe belongs to."""
    rets, lens = [], []
    for p in range(PROBES if probes is None else probes):
        th, a_n, b_n = nudged_inputs(w, theta, a_mat, b_mat, seed=1000 * (int(w.seed) % 1000) + p)
        ret, ln, _, _ = oracle.rollout(w, gen, th, eps, a_n, b_n, individuals=individuals, noise_row0=noise_row0, obs_norm=obs_norm)
        rets.append(ret.astype(np.float64))
        lens.append(ln)
    return np.stack(rets, axis=-1), np.stack(lens, axis=-1)


def spread_of(probe, r_ret, r_len):
    """(spread [n, E], mean_spread, dev [n, E, P]): largest relative deviation of the nudged returns from the reference
    per episode (+inf where a nudge changed the episode's length), the root mean square over the nudge sets of the
    relative shift of the batch-mean return, and the deviations themselves."""
    p_ret, p_len = probe
    r64 = r_ret.astype(np.float64)
    scale = np.maximum(np.abs(r64), 1e-3)
    dev = np.abs(p_ret - r64[..., None]) / scale[..., None]
    dev[p_len != r_len[..., None]] = np.inf
    shifts = []
    for p in range(p_ret.shape[-1]):
        same = p_len[..., p] == r_len
        if same.any():
            shifts.append((float(p_ret[..., p][same].mean()) - float(r64[same].mean())) / max(abs(float(r64[same].mean())), 1e-3))
    return dev.max(axis=-1), (float(np.sqrt(np.mean(np.square(shifts)))) if shifts else float("inf")), dev
