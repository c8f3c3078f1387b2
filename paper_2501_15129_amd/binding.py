"""Thin ctypes binding of the C boundary in ``include/es.h``.

Argument marshalling only: every step of the hot path runs in the HIP kernels of
``libes_hip.so``.  PyTorch supplies device memory (``tensor.data_ptr()``) and the stream.
There is no CPU fallback: if the library is missing, importing fails loudly.
"""
from __future__ import annotations

import ctypes as C
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libes_hip.so"

ES_OK, ES_EINVAL, ES_EUNSUPPORTED, ES_EHIP = 0, -1, -2, -3


class EsConfig(C.Structure):
    """Mirror of ``struct es_config``."""
    _fields_ = [
        ("pop", C.c_uint32), ("envs_per_ind", C.c_uint32), ("horizon", C.c_uint32),
        ("obs_dim", C.c_uint32), ("hid_dim", C.c_uint32), ("act_dim", C.c_uint32),
        ("dtype", C.c_uint32), ("noise_dtype", C.c_uint32),
        ("antithetic", C.c_uint32), ("out_tanh", C.c_uint32),
        ("sigma", C.c_float), ("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float),
        ("adam_eps", C.c_float), ("weight_decay", C.c_float),
        ("done_thresh", C.c_float), ("act_cost", C.c_float),
        ("seed", C.c_uint64),
        ("algorithm", C.c_uint32), ("num_elites", C.c_uint32), ("hidden_act", C.c_uint32), ("num_hidden", C.c_uint32),
        ("noise_table_len", C.c_uint64),
        ("episodes_per_env", C.c_uint32), ("env_dtype", C.c_uint32),
    ]


class EsError(RuntimeError):
    def __init__(self, status: int, name: str, detail: str):
        super().__init__(f"{name} ({detail})" if detail else name)
        self.status = status


def load_library() -> C.CDLL:
    if not _LIB_PATH.exists():
        raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2501_15129_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(str(_LIB_PATH))
    vp, u64, sz = C.c_void_p, C.c_uint64, C.c_size_t
    lib.es_create.argtypes = [C.POINTER(EsConfig), C.POINTER(vp)]
    lib.es_destroy.argtypes = [vp]
    for fn in ("es_param_count", "es_noise_rows", "es_noise_ld", "es_noise_bytes", "es_workspace_bytes"):
        getattr(lib, fn).argtypes = [vp]
        getattr(lib, fn).restype = sz
    lib.es_rollout_kernel.argtypes = [vp]
    lib.es_rollout_kernel.restype = C.c_char_p
    lib.es_update_kernel.argtypes = [vp]
    lib.es_update_kernel.restype = C.c_char_p
    lib.es_strerror.argtypes = [C.c_int]
    lib.es_strerror.restype = C.c_char_p
    lib.es_last_error.argtypes = [vp]
    lib.es_last_error.restype = C.c_char_p
    lib.es_set_obs_norm.argtypes = [vp, vp, vp]
    lib.es_build_noise_table.argtypes = [vp, vp, vp]
    lib.es_sample_population.argtypes = [vp, u64, vp, vp]
    lib.es_rollout.argtypes = [vp, u64, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.es_rank.argtypes = [vp, vp, vp, vp, vp]
    lib.es_update.argtypes = [vp, u64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.es_generation.argtypes = [vp, u64, u64] + [vp] * 14
    lib.es_update_static.argtypes = [vp, u64, vp, vp, vp, vp, vp, vp, vp]
    lib.es_static_scratch_bytes.argtypes = []
    lib.es_static_scratch_bytes.restype = sz
    return lib


_lib = load_library()


def make_config(w) -> EsConfig:
    """Build an ``es_config`` from a workload description (fields of ``workloads.Workload``)."""
    return EsConfig(pop=w.pop, envs_per_ind=w.envs, horizon=w.horizon, obs_dim=w.obs, hid_dim=w.hid,
                    act_dim=w.act, dtype=w.dtype, noise_dtype=w.noise_dtype, antithetic=w.antithetic,
                    out_tanh=w.out_tanh, sigma=w.sigma, lr=w.lr, beta1=w.beta1, beta2=w.beta2,
                    adam_eps=w.adam_eps, weight_decay=w.weight_decay, done_thresh=w.done_thresh,
                    act_cost=w.act_cost, seed=w.seed,
                    algorithm=getattr(w, "algorithm", 0), num_elites=getattr(w, "num_elites", 0),
                    hidden_act=getattr(w, "hidden_act", 0), num_hidden=getattr(w, "num_hidden", 2),
                    noise_table_len=getattr(w, "noise_table_len", 0),
                    episodes_per_env=getattr(w, "episodes", 1), env_dtype=getattr(w, "env_dtype", 0))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t, dtype, numel, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if t.numel() < numel:
        raise ValueError(f"{name}: needs {numel} elements, got {t.numel()}")
    return t.data_ptr()


class EsContext:
    """Owns one ``es_ctx``.  Method names and argument order follow ``include/es.h``."""

    def __init__(self, cfg):
        self.cfg = cfg if isinstance(cfg, EsConfig) else make_config(cfg)
        h = C.c_void_p()
        rc = _lib.es_create(C.byref(self.cfg), C.byref(h))
        if rc != ES_OK:
            raise EsError(rc, _lib.es_strerror(rc).decode(), _lib.es_last_error(None).decode())
        self._h = h
        self.param_count = int(_lib.es_param_count(h))
        self.noise_rows = int(_lib.es_noise_rows(h))
        self.noise_ld = int(_lib.es_noise_ld(h))
        self.noise_bytes = int(_lib.es_noise_bytes(h))
        self.workspace_bytes = int(_lib.es_workspace_bytes(h))
        self.rollout_kernel = _lib.es_rollout_kernel(h).decode()
        self.update_kernel = _lib.es_update_kernel(h).decode()
        self.noise_torch_dtype = torch.bfloat16 if self.cfg.noise_dtype == 1 else torch.float32
        self.noise_regenerated = self.cfg.noise_dtype in (2, 3)     # no matrix: every `noise` argument is None
        self.noise_table = self.cfg.noise_dtype >= 4                # `noise` is a raw byte buffer: table | row offsets
        self.episodes = self.cfg.envs_per_ind * max(1, self.cfg.episodes_per_env)   # E: columns of returns / ep_len

    def close(self):
        if getattr(self, "_h", None) and _lib is not None:      # module globals may be gone at interpreter shutdown
            _lib.es_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def _check(self, rc):
        if rc != ES_OK:
            raise EsError(rc, _lib.es_strerror(rc).decode(), _lib.es_last_error(self._h).decode())

    # -- buffers (plumbing: torch owns the memory) --------------------------------
    def alloc_noise(self, device="cuda"):
        if self.noise_regenerated:
            return None
        if self.noise_table:
            return torch.empty(self.noise_bytes, dtype=torch.uint8, device=device)
        return torch.empty((self.noise_rows, self.noise_ld), dtype=self.noise_torch_dtype, device=device)

    def alloc_workspace(self, device="cuda"):
        return torch.empty(self.workspace_bytes, dtype=torch.uint8, device=device)

    def _noise_ptr(self, noise, n):
        if self.noise_regenerated:
            return None
        if self.noise_table:
            return _ptr(noise, torch.uint8, self.noise_bytes, "noise")
        return _ptr(noise, self.noise_torch_dtype, n, "noise")

    def build_noise_table(self, noise):
        """Fill the shared noise table (noise_dtype 4, 5) once; ``noise`` comes from ``alloc_noise()``."""
        self._check(_lib.es_build_noise_table(self._h, _ptr(noise, torch.uint8, self.noise_bytes, "noise"), _stream()))

    def set_obs_norm(self, mean, inv_std):
        """Frozen observation statistics ([obs] float32 device tensors, kept alive here), or ``None, None``."""
        n = self.cfg.obs_dim
        self._obs_norm = (mean, inv_std)
        self._check(_lib.es_set_obs_norm(self._h, _ptr(mean, torch.float32, n, "mean"),
                                         _ptr(inv_std, torch.float32, n, "inv_std")))

    # -- the four hot calls ---------------------------------------------------------
    def sample_population(self, generation: int, noise):
        n = self.noise_rows * self.noise_ld
        self._check(_lib.es_sample_population(self._h, generation, self._noise_ptr(noise, n),
                                              _stream()))

    def rollout(self, generation: int, theta, noise, a_mat, b_mat, returns, ep_len, fitness, workspace):
        c = self.cfg
        f32, n = torch.float32, self.noise_rows * self.noise_ld
        self._check(_lib.es_rollout(
            self._h, generation, _ptr(theta, f32, self.param_count, "theta"),
            self._noise_ptr(noise, n),
            _ptr(a_mat, f32, c.obs_dim * c.obs_dim, "A"), _ptr(b_mat, f32, c.obs_dim * c.act_dim, "B"),
            _ptr(returns, f32, c.pop * self.episodes, "returns"),
            _ptr(ep_len, torch.int32, c.pop * self.episodes, "ep_len"),
            _ptr(fitness, f32, c.pop, "fitness"),
            _ptr(workspace, torch.uint8, self.workspace_bytes, "workspace"), _stream()))

    def rank(self, fitness, rank, shaped):
        n = self.cfg.pop
        self._check(_lib.es_rank(self._h, _ptr(fitness, torch.float32, n, "fitness"),
                                 _ptr(rank, torch.int32, n, "rank"), _ptr(shaped, torch.float32, n, "shaped"),
                                 _stream()))

    def update(self, adam_step: int, noise, shaped, theta, m, v, grad, workspace):
        f32, d, n = torch.float32, self.param_count, self.noise_rows * self.noise_ld
        self._check(_lib.es_update(
            self._h, adam_step, self._noise_ptr(noise, n),
            _ptr(shaped, f32, self.cfg.pop, "shaped"), _ptr(theta, f32, d, "theta"), _ptr(m, f32, d, "m"),
            _ptr(v, f32, d, "v"), _ptr(grad, f32, d, "grad"),      # m, v may be None for ARS / VanillaES
            _ptr(workspace, torch.uint8, self.workspace_bytes, "workspace"), _stream()))

    def update_static(self, adam_step: int, noise, shaped, theta, m, v, grad):
        """``es_update`` without a workspace argument: partial sums go to the library's built-in scratch."""
        f32, d, n = torch.float32, self.param_count, self.noise_rows * self.noise_ld
        self._check(_lib.es_update_static(
            self._h, adam_step, self._noise_ptr(noise, n),
            _ptr(shaped, f32, self.cfg.pop, "shaped"), _ptr(theta, f32, d, "theta"), _ptr(m, f32, d, "m"),
            _ptr(v, f32, d, "v"), _ptr(grad, f32, d, "grad"), _stream()))

    def generation(self, generation: int, adam_step: int, noise, a_mat, b_mat, theta, m, v, returns, ep_len, fitness,
                   rank, shaped, grad, workspace):
        c = self.cfg
        f32, i32, d, n = torch.float32, torch.int32, self.param_count, self.noise_rows * self.noise_ld
        self._check(_lib.es_generation(
            self._h, generation, adam_step, self._noise_ptr(noise, n),
            _ptr(a_mat, f32, c.obs_dim * c.obs_dim, "A"), _ptr(b_mat, f32, c.obs_dim * c.act_dim, "B"),
            _ptr(theta, f32, d, "theta"), _ptr(m, f32, d, "m"), _ptr(v, f32, d, "v"),
            _ptr(returns, f32, c.pop * self.episodes, "returns"), _ptr(ep_len, i32, c.pop * self.episodes, "ep_len"),
            _ptr(fitness, f32, c.pop, "fitness"), _ptr(rank, i32, c.pop, "rank"), _ptr(shaped, f32, c.pop, "shaped"),
            _ptr(grad, f32, d, "grad"), _ptr(workspace, torch.uint8, self.workspace_bytes, "workspace"), _stream()))


def raw_library() -> C.CDLL:
    """The loaded ``libes_hip.so`` (for tests that exercise the C boundary's error paths)."""
    return _lib
