"""ctypes front end of the CPU checker in ``es_oracle.c``: TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's CPU-baseline leg import this
package.  Nothing here touches the HIP library, and the HIP package never
imports this one.  Arrays are numpy; the noise matrix is dense ``[rows, D]``
float32 (values already rounded to bf16 when the workload stores bf16 noise).
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = [_HERE / "es_oracle.c", _HERE / "rollout_body.inc"]
_LIB = _HERE / "liboracle.so"


class OrcConfig(C.Structure):
    _fields_ = [
        ("pop", C.c_uint32), ("envs", C.c_uint32), ("horizon", C.c_uint32),
        ("obs", C.c_uint32), ("hid", C.c_uint32), ("act", C.c_uint32),
        ("dtype", C.c_uint32), ("noise_dtype", C.c_uint32),
        ("antithetic", C.c_uint32), ("out_tanh", C.c_uint32),
        ("sigma", C.c_float), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
        ("adam_eps", C.c_float), ("weight_decay", C.c_float),
        ("done_thresh", C.c_float), ("act_cost", C.c_float),
        ("seed", C.c_uint64),
        ("hidden_act", C.c_uint32), ("num_hidden", C.c_uint32), ("episodes", C.c_uint32), ("env_dtype", C.c_uint32),
    ]


_LIB_SAN = _HERE / "liboracle_san.so"


def build(force: bool = False, sanitize: bool = False) -> Path:
    """Compile the checker with gcc (contraction off so the binary32 sequences are exact).

    ``sanitize=True`` builds a second library, ``liboracle_san.so``, with AddressSanitizer and
    UndefinedBehaviorSanitizer (host code only); a process that loads it needs the sanitizer runtime
    preloaded (``sanitizer_runtime()``), which is what the sanitizer test's child process does."""
    lib_path = _LIB_SAN if sanitize else _LIB
    stale = (not lib_path.exists()) or any(p.stat().st_mtime > lib_path.stat().st_mtime for p in _SRC)
    if force or stale:
        tmp = lib_path.with_suffix(f".tmp{os.getpid()}.so")
        extra = ["-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"] if sanitize else []
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", *extra,
                               "-o", str(tmp), str(_SRC[0]), "-lm"], cwd=str(_HERE))
        os.replace(tmp, lib_path)
    return lib_path


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime, to be preloaded by a process that loads the sanitized checker."""
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


_lib = None


def lib():
    global _lib
    if _lib is None:
        # ORACLE_SANITIZE=1 (set by the sanitizer test for its child process): the instrumented build
        _lib = C.CDLL(str(build(sanitize=os.environ.get("ORACLE_SANITIZE") == "1")))
        _lib.orc_param_count.restype = C.c_size_t
        _lib.orc_bf16_round.restype = C.c_float
        _lib.orc_bf16_round.argtypes = [C.c_float]
        _lib.orc_max_threads.restype = C.c_int
    return _lib


def config(w) -> OrcConfig:
    """Build the checker's config from a workload description (any object with these fields)."""
    c = OrcConfig()
    for name, _ in OrcConfig._fields_:
        setattr(c, name, getattr(w, name, 0) if name in ("hidden_act", "num_hidden", "episodes", "env_dtype") else getattr(w, name))
    return c


def _p(a, ctype):
    return a.ctypes.data_as(C.POINTER(ctype))


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def max_threads() -> int:
    return int(lib().orc_max_threads())


def set_threads(n: int) -> None:
    """Threads of the checker's OpenMP loops from now on (the benchmark's single-thread leg)."""
    lib().orc_set_threads(C.c_int(int(n)))


def param_count(w) -> int:
    c = config(w)
    return int(lib().orc_param_count(C.byref(c)))


def philox4x32_10(ctr, key):
    c = (C.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (C.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (C.c_uint32 * 4)()
    lib().orc_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def gauss_pair(xa: int, xb: int):
    z = (C.c_float * 2)()
    lib().orc_gauss_pair(C.c_uint32(xa), C.c_uint32(xb), z)
    return float(z[0]), float(z[1])


def bf16_round(x):
    a = np.asarray(x, dtype=np.float32)
    out = np.empty_like(a)
    f = lib().orc_bf16_round
    flat_in, flat_out = a.ravel(), out.ravel()
    for i in range(flat_in.size):
        flat_out[i] = f(float(flat_in[i]))
    return out


def sample_population(w, gen: int, rows=None) -> np.ndarray:
    """Noise rows ``rows=(j0, j1)`` (default: all) of generation ``gen``: float32 ``[j1-j0, D]``."""
    c = config(w)
    d = param_count(w)
    j0, j1 = (0, w.noise_rows) if rows is None else rows
    out = np.empty((j1 - j0, d), dtype=np.float32)
    lib().orc_sample_rows(C.byref(c), C.c_uint64(gen), C.c_uint32(j0), C.c_uint32(j1), _p(out, C.c_float))
    return out


def perturb(w, theta, noise, i: int) -> np.ndarray:
    """Parameters of individual ``i``; ``noise`` is the full dense matrix."""
    c = config(w)
    theta, noise = _f32(theta), _f32(noise)
    row = _f32(noise[i // 2 if w.antithetic else i])
    out = np.empty(param_count(w), dtype=np.float32)
    lib().orc_perturb(C.byref(c), _p(theta, C.c_float), _p(row, C.c_float), C.c_uint32(i), _p(out, C.c_float))
    return out


def reset(w, gen: int, e: int) -> np.ndarray:
    c = config(w)
    out = np.empty(w.obs, dtype=np.float32)
    lib().orc_reset(C.byref(c), C.c_uint64(gen), C.c_uint32(e), _p(out, C.c_float))
    return out


def rollout(w, gen: int, theta, noise, a_mat, b_mat, individuals=None, arith: int = 0, noise_row0: int = 0,
            obs_norm=None):
    """Evaluate individuals ``(i0, i1)`` (default all).  ``noise`` holds the dense rows from
    ``noise_row0`` on (the full matrix by default); it must cover the rows of these individuals.

    ``obs_norm = (mean [obs], inv_std [obs])``: frozen observation statistics for the policy's input.

    Returns ``(returns [n,E*K] f32, ep_len [n,E*K] i32, fitness [n] f32, margin [n,E*K] f32)`` with ``K`` the
    episodes per environment copy (1 unless the workload sets ``episodes``).
    """
    c = config(w)
    theta, noise, a_mat, b_mat = _f32(theta), _f32(noise), _f32(a_mat), _f32(b_mat)
    i0, i1 = (0, w.pop) if individuals is None else individuals
    n = i1 - i0
    first, last = (i0 // 2, (i1 - 1) // 2) if w.antithetic else (i0, i1 - 1)
    assert noise.ndim == 2 and noise.shape[1] == param_count(w)
    assert noise_row0 <= first and last < noise_row0 + noise.shape[0], "noise rows do not cover these individuals"
    cols = w.envs * max(1, getattr(w, "episodes", 1))     # episodes of one environment copy sit next to each other
    ret = np.empty((n, cols), dtype=np.float32)
    ln = np.empty((n, cols), dtype=np.int32)
    fit = np.empty(n, dtype=np.float32)
    mar = np.empty((n, cols), dtype=np.float32)
    null = C.POINTER(C.c_float)()
    mean = inv = None
    if obs_norm is not None:
        mean, inv = _f32(obs_norm[0]), _f32(obs_norm[1])
        assert mean.shape == (w.obs,) and inv.shape == (w.obs,)
    lib().orc_rollout_norm(C.byref(c), C.c_uint64(gen), _p(theta, C.c_float), _p(noise, C.c_float),
                           C.c_uint32(noise_row0), _p(a_mat, C.c_float), _p(b_mat, C.c_float),
                           null if mean is None else _p(mean, C.c_float), null if inv is None else _p(inv, C.c_float),
                           C.c_uint32(i0), C.c_uint32(i1),
                           C.c_int(arith), _p(ret, C.c_float), _p(ln, C.c_int32), _p(fit, C.c_float),
                           _p(mar, C.c_float))
    return ret, ln, fit, mar


def rank(fitness):
    f = _f32(fitness)
    n = f.size
    r = np.empty(n, dtype=np.int32)
    u = np.empty(n, dtype=np.float32)
    lib().orc_rank(C.c_uint32(n), _p(f, C.c_float), _p(r, C.c_int32), _p(u, C.c_float))
    return r, u


def update(w, adam_step: int, noise, shaped, theta, m, v):
    """One gradient-estimate + Adam step.  Returns new ``(theta, m, v, g)`` (inputs untouched)."""
    c = config(w)
    noise, shaped = _f32(noise), _f32(shaped)
    assert noise.shape == (w.noise_rows, param_count(w)) and shaped.size == w.pop
    th, mm, vv = (np.array(x, dtype=np.float32, copy=True) for x in (theta, m, v))
    g = np.empty(param_count(w), dtype=np.float32)
    lib().orc_update(C.byref(c), C.c_uint64(adam_step), _p(noise, C.c_float), _p(shaped, C.c_float),
                     _p(th, C.c_float), _p(mm, C.c_float), _p(vv, C.c_float), _p(g, C.c_float))
    return th, mm, vv, g


def rank_ars(fitness, elites: int):
    """ARS direction selection: ``(rank [N] i32, shaped [N] f32)`` (see ``orc_rank_ars``)."""
    f = _f32(fitness)
    r = np.empty(f.size, dtype=np.int32)
    u = np.empty(f.size, dtype=np.float32)
    lib().orc_rank_ars(C.c_uint32(f.size), C.c_uint32(elites), _p(f, C.c_float), _p(r, C.c_int32), _p(u, C.c_float))
    return r, u


def update_ars(w, elites: int, noise, shaped, theta):
    """ARS step (plain SGD ascent).  Returns new ``(theta, g)``."""
    c = config(w)
    noise, shaped = _f32(noise), _f32(shaped)
    assert noise.shape == (w.pop // 2, param_count(w)) and shaped.size == w.pop
    th = np.array(theta, dtype=np.float32, copy=True)
    g = np.empty(param_count(w), dtype=np.float32)
    lib().orc_update_ars(C.byref(c), C.c_uint32(elites), _p(noise, C.c_float), _p(shaped, C.c_float),
                         _p(th, C.c_float), _p(g, C.c_float))
    return th, g


def rank_vanilla(fitness, elites: int):
    """VanillaES truncation selection with log-rank weights: ``(rank, shaped)``."""
    f = _f32(fitness)
    r = np.empty(f.size, dtype=np.int32)
    u = np.empty(f.size, dtype=np.float32)
    lib().orc_rank_vanilla(C.c_uint32(f.size), C.c_uint32(elites), _p(f, C.c_float), _p(r, C.c_int32), _p(u, C.c_float))
    return r, u


def update_vanilla(w, noise, shaped, theta):
    """VanillaES recombination.  Returns new ``(theta, g)`` with ``g = theta_new - theta``."""
    c = config(w)
    noise, shaped = _f32(noise), _f32(shaped)
    assert noise.shape == (w.pop, param_count(w)) and shaped.size == w.pop and not w.antithetic
    th = np.array(theta, dtype=np.float32, copy=True)
    g = np.empty(param_count(w), dtype=np.float32)
    lib().orc_update_vanilla(C.byref(c), _p(noise, C.c_float), _p(shaped, C.c_float), _p(th, C.c_float), _p(g, C.c_float))
    return th, g


def table_slice(w, t0: int, t1: int, round_bf16: bool) -> np.ndarray:
    """Entries ``t0 <= t < t1`` of the shared noise table (float32)."""
    c = config(w)
    out = np.empty(t1 - t0, dtype=np.float32)
    lib().orc_table_slice(C.byref(c), C.c_uint64(t0), C.c_uint64(t1), C.c_int(1 if round_bf16 else 0), _p(out, C.c_float))
    return out


def table_offsets(w, gen: int, table_len: int, span: int) -> np.ndarray:
    """Start of every noise row of generation ``gen`` in a table of ``table_len`` entries (uint32, multiples of 8)."""
    c = config(w)
    out = np.empty(w.noise_rows, dtype=np.uint32)
    lib().orc_table_offsets(C.byref(c), C.c_uint64(gen), C.c_uint64(table_len), C.c_uint64(span), C.c_uint32(w.noise_rows),
                            _p(out, C.c_uint32))
    return out


def table_rows(w, gen: int, table_len: int, span: int, round_bf16: bool, table=None) -> np.ndarray:
    """Dense ``[rows, D]`` noise matrix of generation ``gen`` read out of the table (for the stages that take a matrix)."""
    d = param_count(w)
    offs = table_offsets(w, gen, table_len, span)
    if table is None:
        table = table_slice(w, 0, table_len, round_bf16)
    return np.stack([table[int(o):int(o) + d] for o in offs]).astype(np.float32)
