"""Seeded synthetic workloads: the five benchmark shapes and their input arrays.

This module only *draws inputs* (environment matrices, the initial parameter
vector, zeroed optimiser moments).  It contains none of the method's arithmetic
(no noise stream, no perturbation, no rollout, no ranking, no optimiser) so
that the HIP path and the CPU checker can both be fed from it without sharing
any code of the method itself.

The environment is a stand-in for the locomotion simulators the paper times
on (Sec. 5.1, fixed-length episodes of 1000 steps; Sec. 5.2 population size and
[256,256] networks): a state vector of locomotion-task width, a dense policy
MLP, a per-step reward and an early-termination rule.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import math

import numpy as np


@dataclass(frozen=True)
class Workload:
    """Static description of one OpenES generation (paper Sec. 3.2, 5.1, App. B Table 5b)."""
    name: str
    pop: int            # N, population size
    envs: int           # E, environment copies (episodes) per individual
    horizon: int        # T, maximum episode length
    obs: int            # n_o
    hid: int            # n_h (two hidden layers)
    act: int            # n_a
    dtype: int          # 0: fp32 ; 1: bf16 contraction operands, fp32 accumulate
    noise_dtype: int    # 0 / 1: fp32 / bf16 noise matrix ; 2 / 3: regenerated ; 4 / 5: rows of a shared fp32 / bf16 table
    seed: int
    sigma: float = 0.02
    lr: float = 0.01
    beta1: float = 0.9
    beta2: float = 0.999
    adam_eps: float = 1e-8
    weight_decay: float = 0.005
    done_thresh: float = 0.95
    act_cost: float = 0.01
    antithetic: int = 1
    out_tanh: int = 1
    algorithm: int = 0  # 0 OpenES ; 1 ARS ; 2 VanillaES (paper Sec. 4)
    num_elites: int = 0 # ARS: directions kept ; VanillaES: parents
    hidden_act: int = 0 # hidden-layer activation: 0 tanh ; 1 ReLU (paper App. B)
    num_hidden: int = 2 # m hidden layers of width hid (paper Sec. 5.1 varies m; base case 2)
    noise_table_len: int = 0  # entries of the shared noise table (noise_dtype 4, 5; paper Sec. 5.1)
    episodes: int = 1   # episodes run back to back in every environment copy (auto-reset; paper Sec. 3.1)
    env_dtype: int = 0  # with dtype 1: 0 = the environment's products use bf16 operands too ; 1 = the environment stays binary32
    # input recipe only (seen by make_inputs, not by the library or the checker):
    a_radius: float = 0.9       # spectral radius the environment matrix A is rescaled to
    b_var: float = 1.0 / 3.0    # variance of the entries of B
    bias_std: float = 0.0       # standard deviation of the initial biases (0: biases start at zero)

    @property
    def n_params(self) -> int:
        o, h, a, m = self.obs, self.hid, self.act, self.num_hidden
        return (o + 1) * h + (m - 1) * (h + 1) * h + (h + 1) * a

    @property
    def noise_rows(self) -> int:
        return self.pop // 2 if self.antithetic else self.pop

    @property
    def env_steps(self) -> int:
        return self.pop * self.envs * self.episodes * self.horizon

    def fixed_length(self) -> "Workload":
        """Same workload with the termination rule switched off (every episode runs T steps)."""
        return replace(self, name=self.name + "-fixedlen", done_thresh=math.inf)

    def contractive(self) -> "Workload":
        """Twin of this workload - same population, copies, horizon, widths, precision, fixed-length
        episodes (the paper's timing protocol, Sec. 5.1) - whose closed loop s' = tanh(A s + B pi(s)) is a
        contraction: A and B are drawn from the same streams and scaled down, and the policy starts with
        non-zero biases so that every individual settles at its own non-trivial fixed point.  Rounding
        differences between two evaluations of such a loop die out instead of growing, so the returns of a
        finite-precision evaluation can be held to the strict tolerance at the full horizon."""
        return replace(self, name=self.name + "-contractive", done_thresh=math.inf,
                       a_radius=CONTRACTIVE_A_RADIUS, b_var=CONTRACTIVE_B_VAR, bias_std=CONTRACTIVE_BIAS_STD)


# Scales of the contractive twins (chosen by measurement on the CPU checker alone: one-ulp nudges of a
# handful of operands move no return of any twin by more than 1/8 of its tolerance at T = 1000).
CONTRACTIVE_A_RADIUS = 0.5
CONTRACTIVE_B_VAR = 0.1
CONTRACTIVE_BIAS_STD = 0.3

CONFIGS = (
    Workload("cfg0", pop=8, envs=4, horizon=100, obs=11, hid=32, act=3, dtype=0, noise_dtype=0, seed=0),
    Workload("cfg1", pop=16, envs=16, horizon=1000, obs=17, hid=64, act=6, dtype=0, noise_dtype=0, seed=1),
    Workload("cfg2", pop=256, envs=1, horizon=1000, obs=17, hid=64, act=6, dtype=0, noise_dtype=0, seed=2),
    Workload("cfg3", pop=1024, envs=16, horizon=1000, obs=27, hid=256, act=8, dtype=1, noise_dtype=1, seed=3),
    Workload("cfg4", pop=4096, envs=4, horizon=1000, obs=244, hid=256, act=17, dtype=1, noise_dtype=1, seed=4),
)


def layer_shapes(w: Workload):
    """Shapes of W1, b1, (W_l, b_l for the further hidden layers), W3, b3 in flat-parameter order;
    matrices are [out, in] row-major."""
    o, h, a = w.obs, w.hid, w.act
    return ((h, o), (h,)) + ((h, h), (h,)) * (w.num_hidden - 1) + ((a, h), (a,))


def make_inputs(w: Workload):
    """Draw A [n_o,n_o], B [n_o,n_a], theta0 [D] (float32) for a workload, from its seed.

    A: i.i.d. N(0,1) rescaled to spectral radius ``a_radius`` (0.9).  B: i.i.d. N(0, ``b_var``) (1/3).
    theta0: every weight matrix N(0, 2/(fan_in+fan_out)), biases zero (N(0, ``bias_std``^2) for the
    contractive twins).
    """
    rng = np.random.default_rng([int(w.seed), 0x45534D49])
    g = rng.standard_normal((w.obs, w.obs))
    rho = float(np.max(np.abs(np.linalg.eigvals(g))))
    a_mat = (w.a_radius / rho) * g
    b_mat = rng.standard_normal((w.obs, w.act)) * math.sqrt(w.b_var)
    parts = []
    bias_rng = np.random.default_rng([int(w.seed), 0x42494153])     # a stream of its own: the weights do not move
    for shp in layer_shapes(w):
        if len(shp) == 2:
            fan_out, fan_in = shp
            parts.append((rng.standard_normal(shp) * math.sqrt(2.0 / (fan_in + fan_out))).ravel())
        else:
            parts.append(bias_rng.standard_normal(shp) * w.bias_std if w.bias_std else np.zeros(shp))
    theta0 = np.concatenate(parts)
    assert theta0.size == w.n_params
    return (np.ascontiguousarray(a_mat, dtype=np.float32),
            np.ascontiguousarray(b_mat, dtype=np.float32),
            np.ascontiguousarray(theta0, dtype=np.float32))


def random_fitness(n: int, seed: int, ties: bool = False) -> np.ndarray:
    """A seeded fitness vector for exercising the ranking / update stages on their own."""
    rng = np.random.default_rng([seed, 0x46495421])
    f = rng.standard_normal(n).astype(np.float32) * 100.0
    if ties and n >= 4:
        f[rng.integers(0, n, size=n // 4)] = f[0]
    return f
