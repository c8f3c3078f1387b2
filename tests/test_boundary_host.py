"""Host-side checks of the C boundary that need no GPU: the library loads, exports every
symbol the header declares, validates configurations and rejects bad arguments before
any launch."""
import ctypes as C
import math
import re
from dataclasses import replace
from pathlib import Path

import pytest

from paper_2501_15129_amd.workloads import CONFIGS, Workload

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def binding():
    from paper_2501_15129_amd import binding as b
    return b


def test_library_exports_every_declared_symbol(binding):
    header = (ROOT / "include" / "es.h").read_text()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(es_[a-z_]+)\s*\(", body))
    assert {"es_create", "es_destroy", "es_sample_population", "es_rollout", "es_rank", "es_update", "es_generation"} <= declared
    lib = binding.raw_library()
    for name in sorted(declared):
        assert hasattr(lib, name), f"libes_hip.so does not export {name}"


def test_config_struct_matches_header(binding):
    header = (ROOT / "include" / "es.h").read_text()
    struct = header[header.index("typedef struct es_config {"):header.index("} es_config;")]
    struct = re.sub(r"/\*.*?\*/", "", struct, flags=re.S)
    names = []
    for decl in re.findall(r"(?:uint32_t|uint64_t|float)\s+([^;]+);", struct):
        names += [n.strip() for n in decl.split(",")]
    assert names == [n for n, _ in binding.EsConfig._fields_]
    assert C.sizeof(binding.EsConfig) == 112       # 10 u32 + 8 f32 + u64 + 4 u32 + u64 + u32 + padding


def test_context_queries(binding):
    for w, d in zip(CONFIGS, (1539, 5702, 5702, 75016, 132881)):
        ctx = binding.EsContext(w)
        assert ctx.param_count == d
        assert ctx.noise_rows == w.pop // 2
        assert ctx.noise_ld >= d and ctx.noise_ld % 512 == 0 and ctx.noise_ld - d < 512
        assert ctx.noise_bytes == ctx.noise_rows * ctx.noise_ld * (2 if w.noise_dtype else 4)
        assert ctx.workspace_bytes >= 256
        assert ctx.rollout_kernel
        ctx.close()


def test_regenerated_noise_contexts_store_nothing(binding):
    from dataclasses import replace
    for mode in (2, 3):
        ctx = binding.EsContext(replace(CONFIGS[4], noise_dtype=mode))
        assert ctx.noise_bytes == 0 and ctx.noise_regenerated and ctx.alloc_noise() is None
        assert ctx.noise_rows == CONFIGS[4].pop // 2                  # the rows still exist, as counters
        assert ctx.update_kernel.startswith("grad_regen_kernel")
        assert ctx.workspace_bytes >= 8 * ctx.noise_ld                # at least one binary64 partial row
        ctx.close()


@pytest.mark.parametrize("bad", [
    dict(pop=7), dict(pop=0), dict(envs=0), dict(horizon=0), dict(obs=0), dict(hid=0), dict(act=0),
    dict(dtype=2), dict(noise_dtype=6), dict(noise_dtype=4, noise_table_len=12), dict(noise_dtype=5, noise_table_len=1024), dict(algorithm=3), dict(hidden_act=2), dict(num_hidden=65), dict(algorithm=1, num_elites=0),
    dict(algorithm=1, num_elites=5, antithetic=0), dict(algorithm=2, num_elites=4), dict(algorithm=2, antithetic=0, num_elites=10**6),
    dict(antithetic=2), dict(out_tanh=5),
    dict(sigma=-1.0), dict(sigma=math.nan), dict(beta1=1.0), dict(beta2=-0.1), dict(adam_eps=0.0),
    dict(done_thresh=math.nan), dict(lr=math.inf),
])
def test_create_rejects_invalid_config(binding, bad):
    with pytest.raises(binding.EsError) as ei:
        binding.EsContext(replace(CONFIGS[0], **bad))
    assert ei.value.status == binding.ES_EINVAL


def test_hot_calls_reject_bad_arguments_before_launch(binding):
    lib = binding.raw_library()
    ctx = binding.EsContext(CONFIGS[0])
    h = ctx._h
    one = C.c_void_p(0x1000)     # never dereferenced: validation fails first
    assert lib.es_sample_population(h, 0, None, None) == binding.ES_EINVAL
    assert lib.es_sample_population(h, 1 << 32, one, None) == binding.ES_EINVAL
    assert lib.es_rank(h, None, one, one, None) == binding.ES_EINVAL
    assert lib.es_rollout(h, 0, one, one, one, one, one, one, None, one, None) == binding.ES_EINVAL
    assert lib.es_update(h, 0, one, one, one, one, one, None, one, None) == binding.ES_EINVAL   # step is 1-based
    assert lib.es_update(h, 1, one, None, one, one, one, None, one, None) == binding.ES_EINVAL
    assert b"adam_step" in lib.es_last_error(h) or b"null" in lib.es_last_error(h)
    zero_sigma = binding.EsContext(replace(CONFIGS[0], sigma=0.0))
    assert lib.es_update(zero_sigma._h, 1, one, one, one, one, one, None, one, None) == binding.ES_EINVAL
    assert lib.es_sample_population(None, 0, one, None) == binding.ES_EINVAL
    assert b"ES_EINVAL" in lib.es_strerror(binding.ES_EINVAL)
    assert b"ES_OK" in lib.es_strerror(0)


def test_hot_calls_reject_misaligned_vector_operands(binding):
    """theta_d, noise_d, A_d, B_d, workspace_d are read with 16-byte loads: a 4-byte-aligned sub-view is refused."""
    lib = binding.raw_library()
    ctx = binding.EsContext(CONFIGS[0])
    h = ctx._h
    ok, off = C.c_void_p(0x1000), C.c_void_p(0x1004)
    args = [ok] * 8          # theta, noise, A, B, returns, ep_len, fitness, workspace
    for k in (0, 1, 2, 3, 7):
        bad = list(args)
        bad[k] = off
        assert lib.es_rollout(h, 0, *bad, None) == binding.ES_EINVAL, k
        assert b"16-byte aligned" in lib.es_last_error(h)
    assert lib.es_sample_population(h, 0, off, None) == binding.ES_EINVAL
    assert lib.es_update(h, 1, off, ok, ok, ok, ok, None, ok, None) == binding.ES_EINVAL
    assert lib.es_update(h, 1, ok, ok, ok, ok, ok, None, off, None) == binding.ES_EINVAL
    # returns / ep_len / fitness only need the alignment of their element type
    assert b"16-byte aligned" in lib.es_last_error(h)


def test_binding_rejects_non_device_tensors(binding):
    import torch
    ctx = binding.EsContext(CONFIGS[0])
    with pytest.raises(TypeError):
        ctx.rank(torch.zeros(8), torch.zeros(8, dtype=torch.int32), torch.zeros(8))


def test_oversized_shape_reports_unsupported_or_picks_a_kernel(binding):
    # a policy far beyond on-chip capacity must be refused cleanly by es_rollout (host check)
    w = Workload("huge", pop=2, envs=1, horizon=1, obs=512, hid=1024, act=64, dtype=0, noise_dtype=0, seed=0)
    ctx = binding.EsContext(w)
    lib = binding.raw_library()
    one = C.c_void_p(0x1000)
    assert lib.es_rollout(ctx._h, 0, one, one, one, one, one, one, one, one, None) == binding.ES_EUNSUPPORTED
    assert b"exceed" in lib.es_last_error(ctx._h)


def test_generated_dpp_runs_are_current():
    """csrc/dpp_runs.inc is the committed output of csrc/gen_dpp_runs.py."""
    import importlib.util
    csrc = ROOT / "paper_2501_15129_amd" / "csrc"
    committed = (csrc / "dpp_runs.inc").read_text()
    spec = importlib.util.spec_from_file_location("gen_dpp_runs", csrc / "gen_dpp_runs.py")
    gen = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(gen)
    gen.main()
    assert (csrc / "dpp_runs.inc").read_text() == committed
