"""Build the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor
from pathlib import Path

HERE = Path(__file__).resolve().parent
CSRC = HERE / "csrc"
LIB = HERE / "libes_hip.so"
MICRO_LIB = HERE / "libes_microbench.so"
SOURCES = ["api.hip", "sample.hip", "rank.hip", "update.hip", "rollout_wave.hip", "rollout_wave_reg.hip",
           "rollout_mfma.hip", "rollout_mfma_f32.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off",
    "-fhip-fp32-correctly-rounded-divide-sqrt",
    # packed-FP32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # MFMA accumulators in architectural VGPRs: the accumulation-register half of the file is
    # reserved for the register-resident policy weights of the rollout kernel
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _compile(src: str) -> Path:
    obj = CSRC / (Path(src).stem + ".o")
    extra = os.environ.get("ES_EXTRA_HIPCC_FLAGS", "").split()      # tuning experiments only
    cmd = [HIPCC, *FLAGS, *extra, "-c", str(CSRC / src), "-o", str(obj)]
    subprocess.check_call(cmd, cwd=str(CSRC))
    return obj


def build(verbose: bool = True) -> Path:
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        objs = list(ex.map(_compile, SOURCES))
    tmp = LIB.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", str(tmp), *map(str, objs)])
    os.replace(tmp, LIB)
    # rate micro-benchmarks (bench.py --peaks): a library of their own, not part of the boundary
    tmp = MICRO_LIB.with_suffix(f".tmp{os.getpid()}.so")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", "-shared", "-o", str(tmp),
                           str(CSRC / "microbench.hip")])
    os.replace(tmp, MICRO_LIB)
    if verbose:
        print(f"built {LIB} and {MICRO_LIB}", file=sys.stderr)
    return LIB


if __name__ == "__main__":
    build()
