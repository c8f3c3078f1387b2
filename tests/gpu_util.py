"""Helpers shared by the GPU parity tests: marshal the checker's dense arrays into the
layouts the C boundary expects, run stages, and compare under the stated tolerances."""
from __future__ import annotations

import numpy as np
import torch

# Target tolerances: episode returns within 1e-4 relative in fp32 and 2e-2 in bf16;
# updated parameters within 1e-5 relative (+1e-7 absolute for parameters near zero).
RET_RTOL = {0: 1e-4, 1: 2e-2}
# |max|s| - done_thresh| below this at any executed step marks an episode whose termination
# step may legitimately differ between binary64 and binary32 / bf16 evaluation.
KNIFE_EDGE = {0: 1e-5, 1: 1e-2}
PARAM_RTOL, PARAM_ATOL = 1e-5, 1e-7


def noise_to_device(ctx, eps_dense: np.ndarray) -> torch.Tensor:
    """Dense float32 [rows, D] (already bf16-valued when the workload stores bf16) -> padded device matrix."""
    rows, d = eps_dense.shape
    assert rows == ctx.noise_rows and d == ctx.param_count
    pad = np.zeros((rows, ctx.noise_ld), dtype=np.float32)
    pad[:, :d] = eps_dense
    t = torch.from_numpy(pad)
    if ctx.cfg.noise_dtype == 1:
        bits = (pad.view(np.uint32) >> 16).astype(np.uint16)
        assert np.array_equal((bits.astype(np.uint32) << 16).view(np.float32), pad), "noise is not bf16-valued"
        t = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16)
    return t.cuda()


def noise_from_device(ctx, noise: torch.Tensor) -> np.ndarray:
    """Device noise matrix -> float32 [rows, ld] on the host (exact widening for bf16)."""
    return noise.detach().float().cpu().numpy()


def dev(x, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype is not None:
        t = t.to(dtype)
    return t.cuda()


def run_rollout(ctx, w, gen, theta, noise_dev, a_mat, b_mat):
    ret = torch.full((w.pop, ctx.episodes), float("nan"), dtype=torch.float32, device="cuda")
    ln = torch.full((w.pop, ctx.episodes), -1, dtype=torch.int32, device="cuda")
    fit = torch.full((w.pop,), float("nan"), dtype=torch.float32, device="cuda")
    ws = ctx.alloc_workspace()
    ctx.rollout(gen, dev(theta), noise_dev, dev(a_mat), dev(b_mat), ret, ln, fit, ws)
    torch.cuda.synchronize()
    return ret.cpu().numpy(), ln.cpu().numpy(), fit.cpu().numpy()


# A trajectory is called sensitive when the checker's OWN second evaluation of it (same
# algorithm, binary32 accumulation instead of binary64) already drifts from the reference by
# more than this fraction of the tolerance: some random policies make the closed loop
# chaotic, and there no finite-precision kernel can track the binary64 return (in bf16 mode a
# single flipped rounding decorrelates the trajectories).  Such episodes are held to
# SENSITIVE_RTOL instead, and the share of episodes that actually need the allowance is capped
# - unless the whole batch is in the chaotic regime (more than CHAOTIC_SHARE of its episodes
# flagged): then every episode is held to SENSITIVE_RTOL, the batch mean to CHAOTIC_MEAN_RTOL,
# and the caller must ALSO pass a strict comparison at a horizon short enough for the
# trajectories not to have diverged (the per-step code path is the same for every step).
SENSITIVE_FRACTION_OF_RTOL = 0.125
SENSITIVE_RTOL = 5e-2
MAX_SENSITIVE_SHARE = 0.03
CHAOTIC_SHARE = 0.25
CHAOTIC_MEAN_RTOL = 1.5e-2


def compare_rollout(w, got, ref, label="", probe=None):
    """got = (returns, ep_len, fitness) from the GPU; ref = (returns, ep_len, fitness, margin) from the
    checker in binary64; probe = the checker's binary32 evaluation of the same episodes (optional).

    Episode lengths must be identical except for episodes the checker flags as knife-edge;
    returns are compared where the lengths agree; fitness where every episode of the
    individual agrees.  Returns (knife-edge flips, worst error on regular episodes,
    number of sensitive episodes, chaotic-regime flag)."""
    g_ret, g_len, g_fit = got
    r_ret, r_len, r_fit, r_mar = ref
    rtol = RET_RTOL[w.dtype]
    scale = np.maximum(np.abs(r_ret), 1e-3)
    if probe is not None:
        sens = (np.abs(probe[0].astype(np.float64) - r_ret) / scale > SENSITIVE_FRACTION_OF_RTOL * rtol) | (probe[1] != r_len)
    else:
        sens = np.zeros(r_ret.shape, dtype=bool)
    chaotic = bool(np.mean(sens) > CHAOTIC_SHARE)
    if chaotic:
        sens = np.ones_like(sens)
    edge = (r_mar < KNIFE_EDGE[w.dtype]) | sens
    same = g_len == r_len
    assert np.all(same | edge), f"{label}: episode length differs away from the termination threshold: " \
        f"{np.argwhere(~(same | edge))[:5].tolist()}"
    # a flagged episode flips only if the two evaluations differ by more than its margin at that step
    assert np.sum(~same) <= 0.3 * np.sum(edge) + 2, \
        f"{label}: too many knife-edge flips ({np.sum(~same)} of {int(np.sum(edge))} flagged, {same.size} episodes)"
    err = np.abs(g_ret.astype(np.float64) - r_ret) / scale
    worst = float(np.max(np.where(same & ~sens, err, 0.0)))
    assert worst <= rtol, f"{label}: return mismatch {worst:.3e} > {rtol}"
    worst_sens = float(np.max(np.where(same & sens, err, 0.0)))
    assert worst_sens <= SENSITIVE_RTOL, f"{label}: return mismatch {worst_sens:.3e} on a sensitive episode"
    if chaotic:
        mean_err = abs(float(np.mean(g_ret[same].astype(np.float64))) - float(np.mean(r_ret[same]))) / abs(float(np.mean(r_ret[same])))
        assert mean_err <= CHAOTIC_MEAN_RTOL, f"{label}: mean return over the batch off by {mean_err:.3e}"
    else:
        excused = same & sens & (err > rtol)
        assert np.mean(excused) <= MAX_SENSITIVE_SHARE + 1.0 / same.size, \
            f"{label}: {int(excused.sum())} sensitive episodes beyond the regular tolerance"
    ind_ok = np.all(same & ~sens, axis=1)
    ferr = np.abs(g_fit.astype(np.float64) - r_fit) / np.maximum(np.abs(r_fit), 1e-3)
    assert float(np.max(np.where(ind_ok, ferr, 0.0))) <= rtol, f"{label}: fitness mismatch"
    # fitness is the mean of the returns the kernel itself produced
    assert np.allclose(g_fit, g_ret.astype(np.float64).mean(axis=1), rtol=1e-5, atol=1e-5), f"{label}: fitness != mean"
    return int(np.sum(~same)), (worst_sens if chaotic else worst), int(sens.sum()), chaotic


def assert_params_close(got, ref, label=""):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bad = np.abs(got - ref) > PARAM_RTOL * np.abs(ref) + PARAM_ATOL
    assert not bad.any(), f"{label}: {int(bad.sum())} of {bad.size} elements off; worst " \
        f"{float(np.max(np.abs(got - ref))):.3e}"
