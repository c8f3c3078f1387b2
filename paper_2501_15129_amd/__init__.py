"""MI355X-native OpenES hot path (population rollout + ES update) behind a C boundary."""
from .workloads import CONFIGS, Workload, make_inputs  # noqa: F401


def __getattr__(name):
    # the binding loads the HIP library on first use and raises if it has not been built
    if name in ("EsContext", "EsConfig", "EsError", "make_config", "raw_library"):
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)
