#!/usr/bin/env python3
"""Benchmark of the OpenES hot path on one MI355X.

One "step" is one whole generation: es_sample_population -> es_rollout -> es_rank ->
es_update, enqueued on one stream with every input already resident in HBM.  The default
workload is the largest configuration (configs[4]: population 4096 x 4 environment copies,
T = 1000, MLP 244-256-256-17, bf16) under the paper's timing protocol of fixed-length
episodes (Sec. 5.1); the same workload with its termination rule switched on is reported
beside it.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from dataclasses import replace
from pathlib import Path

ROOT = Path(__file__).resolve().parent
if str(ROOT) not in sys.path:
    sys.path.insert(0, str(ROOT))

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 MFMA
FP32_VALU_PEAK_TFLOPS = 157.3   # 256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 flop x 2.4 GHz
VALU_PEAK_TLANEOPS = 78.6       # the same figure as vector-lane operations per second (one FMA = one operation)
REGEN_VALU_OPS_PER_BLOCK = 245  # vector instructions per Philox block + two Gaussian transforms + four fp64 FMAs (counted in the built kernel)


def flop_per_env_step(w) -> int:
    """Multiply-add flops of one policy forward plus one environment step (2 flop per MAC)."""
    o, h, a = w.obs, w.hid, w.act
    return 2 * (o * h + (w.num_hidden - 1) * h * h + h * a) + 2 * (o * o + o * a)


def update_bytes(w, ctx) -> int:
    """Algorithmic bytes of es_update: the noise matrix once, theta/m/v read and written, the weights."""
    elt = 2 if w.noise_dtype in (1, 5) else 4
    return w.noise_rows * w.n_params * elt + 24 * w.n_params + 4 * w.pop


def measured_traffic(workload_name: str):
    """HBM bytes per launch measured offline with rocprofv3 (see profiles/), or None for other workloads."""
    f = ROOT / "profiles" / f"hbm_traffic_{workload_name.replace('-', '_')}.txt"
    if not f.exists():
        return None
    for line in f.read_text().splitlines():
        if line.strip() and not line.startswith("#"):
            return json.loads(line)
    return None


def run_generations(torch, ctx, w, bufs, steps, warmup, gen0=0):
    """Runs warmup + steps generations; returns (wall seconds for `steps`, per-stage ms lists, live env steps)."""
    names = ("sample", "rollout", "rank", "update")
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(steps)]
    live = 0

    def generation(g, marks=None):
        if marks: marks[0].record()
        ctx.sample_population(g, bufs["noise"])
        if marks: marks[1].record()
        ctx.rollout(g, bufs["theta"], bufs["noise"], bufs["A"], bufs["B"], bufs["ret"], bufs["len"], bufs["fit"], bufs["ws"])
        if marks: marks[2].record()
        ctx.rank(bufs["fit"], bufs["rank"], bufs["shaped"])
        if marks: marks[3].record()
        ctx.update(g + 1, bufs["noise"], bufs["shaped"], bufs["theta"], bufs["m"], bufs["v"], None, bufs["ws"])
        if marks: marks[4].record()

    for k in range(warmup):
        generation(gen0 + k)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(steps):
        generation(gen0 + warmup + k, ev[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    live = int(bufs["len"].sum().item())            # episode lengths of the last generation
    stage = {n: [ev[k][j].elapsed_time(ev[k][j + 1]) for k in range(steps)] for j, n in enumerate(names)}
    return wall, stage, live


def cpu_model() -> str:
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(w, budget_s=12.0, obs_norm=None, full=False):
    """The CPU checker, as it stands, on the host cores of this machine: a bounded sample of the same workload by
    default (said so in the result), the whole population once with full=True.  Small workloads (under a
    second of checker time) are run whole, and once more on a single thread."""
    import numpy as np
    import oracle
    from paper_2501_15129_amd.workloads import make_inputs

    threads = oracle.max_threads()
    a_mat, b_mat, theta = make_inputs(w)

    def timed(n_ind):
        ws = replace(w, pop=n_ind, noise_dtype=w.noise_dtype & 1)     # the checker's arithmetic does not depend on where the noise is kept
        t0 = time.perf_counter()
        eps = oracle.sample_population(ws, 0)
        ret, ln, fit, _ = oracle.rollout(ws, 0, theta, eps, a_mat, b_mat, obs_norm=obs_norm)
        if ws.algorithm == 1:
            b = max(1, min(ws.num_elites, n_ind // 2))
            oracle.update_ars(ws, b, eps, oracle.rank_ars(fit, b)[1], theta)
        elif ws.algorithm == 2:
            oracle.update_vanilla(ws, eps, oracle.rank_vanilla(fit, max(1, min(ws.num_elites, n_ind)))[1], theta)
        else:
            _, shaped = oracle.rank(fit)
            oracle.update(ws, 1, eps, shaped, theta, np.zeros_like(theta), np.zeros_like(theta))
        return time.perf_counter() - t0, int(ln.sum())

    n = w.pop if full else min(w.pop, 2 * ((threads + 1) // 2))
    dt, steps = timed(n)
    if dt < budget_s and n < w.pop:
        n2 = min(w.pop, 2 * int(max(1, (budget_s / max(dt, 1e-3)) * n / 2)))
        if n2 > n:
            n = n2
            dt, steps = timed(n)
    whole = n == w.pop
    out = {"value": steps / dt, "unit": "env-steps/s", "cores": threads, "kind": "oracle", "cpu_model": cpu_model(),
           "is_sample": not whole, "sampled_fraction_of_population": n / w.pop, "seconds": dt,
           "sample": (f"the WHOLE population, one full generation (sample, rollout, rank, update): {w.pop} individuals" if whole else
                      f"a SAMPLE, not the whole job: one full generation (sample, rollout, rank, update) of the first {n} of {w.pop} individuals")
                     + f" x {w.envs} envs x T={w.horizon}, {steps} env-steps in {dt:.1f} s, OpenMP over individuals on {threads} threads"
                     + ("" if whole else "; bench.py --cpu-full runs all of it")}
    if whole and dt < 5.0:          # the small workloads: also on one thread
        oracle.set_threads(1)
        try:
            dt1, steps1 = timed(n)
        finally:
            oracle.set_threads(threads)
        out["single_thread"] = {"value": steps1 / dt1, "unit": "env-steps/s", "seconds": dt1}
    return out


def measured_peaks(iters=4096):
    """Runs the rate micro-benchmarks of csrc/microbench.hip (every CU, one workgroup each) and returns their figures."""
    import ctypes as C
    lib = C.CDLL(str(ROOT / "paper_2501_15129_amd" / "libes_microbench.so"))
    lib.es_microbench_name.restype = C.c_char_p
    lib.es_microbench_unit.restype = C.c_char_p
    rows = []
    for k in range(lib.es_microbench_count()):
        cyc, ms, rate = C.c_double(), C.c_double(), C.c_double()
        rc = lib.es_microbench_run(k, iters, C.byref(cyc), C.byref(ms), C.byref(rate))
        if rc != 0:
            raise RuntimeError(f"micro-benchmark {k} failed with HIP error {rc}")
        rows.append({"test": lib.es_microbench_name(k).decode(), "unit": lib.es_microbench_unit(k).decode(),
                     "cycles_per_unit_one_wavefront": cyc.value, "launch_ms": ms.value, "chip_units_per_s": rate.value})
    return rows


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", type=int, default=4, help="index into the five workloads (default: the largest)")
    ap.add_argument("--done-rule", action="store_true", help="time the workload with its termination rule on")
    ap.add_argument("--noise-dtype", type=int, default=None, choices=[0, 1, 2, 3, 4, 5],
                    help="override the workload's noise storage: 0/1 stored binary32/bf16 matrix, 2/3 no matrix, values "
                         "regenerated from the counter stream in es_rollout and es_update, 4/5 rows read from a shared "
                         "binary32/bf16 table built once (paper Sec. 5.1)")
    ap.add_argument("--table-len", type=int, default=1 << 26, help="entries of the shared noise table (--noise-dtype 4, 5)")
    ap.add_argument("--algorithm", choices=["openes", "ars", "vanilla"], default="openes",
                    help="strategy of es_rank / es_update (paper Sec. 4); ars and vanilla keep pop/8 elites "
                         "(the ratio of App. B Table 5) and use that table's step sizes")
    ap.add_argument("--hidden-act", choices=["tanh", "relu"], default="tanh",
                    help="hidden-layer activation (the paper's EA experiments use ReLU MLPs, App. B)")
    ap.add_argument("--obs-norm", action="store_true",
                    help="frozen observation statistics for the policy input (paper App. B); synthetic: mean N(0, 0.05^2), std U[0.33, 1]")
    ap.add_argument("--paper-base", action="store_true",
                    help="the base configuration of the paper's OpenES timing experiment (Sec. 5.1: m = 2 hidden layers of 256, "
                         "population n = 128, k = 1 episode, T = 1000) on the synthetic environment at Swimmer's widths (obs 8, act 2), "
                         "bf16 operands; vary it with --num-hidden (m), --pop (n), --episodes-per-env (k)")
    ap.add_argument("--dtype", choices=["bf16", "f32"], default="bf16",
                    help="with --paper-base: bf16 operands (default) or binary32 throughout (fp32 matrix-core kernel)")
    ap.add_argument("--pop", type=int, default=None, help="population size override (with --paper-base: n)")
    ap.add_argument("--num-hidden", type=int, default=2, help="m hidden layers (paper Sec. 5.1 varies m); not the default workload")
    ap.add_argument("--episodes-per-env", type=int, default=1,
                    help="k episodes per environment copy (auto-reset wrapper, paper Sec. 3.1); not the default workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-full", action="store_true",
                    help="run the CPU checker once over the WHOLE population instead of a bounded sample (about two minutes at configs[4])")
    ap.add_argument("--env-f32", action="store_true",
                    help="bf16 workloads: keep the environment's products A s + B a in binary32 (env_dtype = 1; obs <= 64)")
    ap.add_argument("--no-antithetic", action="store_true",
                    help="independent noise rows for every individual (antithetic = 0): at configs[4] es_update then streams the literal "
                         "4096 x 132k bf16 matrix, 1.09 GB")
    ap.add_argument("--no-second-variant", action="store_true", help="skip the extra timing with the termination rule on")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run plain device copies of a known size instead (reference for the HBM byte counters)")
    ap.add_argument("--peaks", action="store_true",
                    help="run the rate micro-benchmarks instead (matrix-core and vector-ALU issue, their overlap, transcendentals, "
                         "LDS, barriers) and print them as one JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build targets one GPU; --gpus N with N > 1 is not supported "
              "(sharding along the population is a design note only)", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2501_15129_amd import CONFIGS, EsContext, make_inputs
    from paper_2501_15129_amd.workloads import Workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    torch.cuda.set_device(0)
    if args.peaks:
        rows = measured_peaks()
        mfma = rows[0]["chip_units_per_s"] * 2 * 16 * 16 * 32 / 1e12
        fma = rows[3]["chip_units_per_s"] * 64 * 2 / 1e12
        print(json.dumps({"peaks": rows, "derived": {"bf16_mfma_tflops_one_wavefront_per_simd": mfma, "published_bf16_mfma_tflops": MFMA_BF16_PEAK_TFLOPS,
                                                     "fp32_fma_tflops_one_wavefront_per_simd": fma, "published_fp32_vector_tflops": FP32_VALU_PEAK_TFLOPS}}))
        return 0
    if args.copy_calibration:
        n_bytes = 1 << 30
        src = torch.empty(n_bytes, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": True, "bytes_read_per_copy": n_bytes, "bytes_written_per_copy": n_bytes,
                          "copies": 3}))
        return 0
    base = CONFIGS[args.config]
    if args.paper_base:
        base = Workload("paper-base", pop=128, envs=1, horizon=1000, obs=8, hid=256, act=2, dtype=1, noise_dtype=1, seed=5)
        if args.dtype == "f32":
            base = replace(base, name="paper-base-f32", dtype=0, noise_dtype=0)
    if args.pop is not None:
        base = replace(base, name=base.name + f"-n{args.pop}", pop=args.pop)
    if args.noise_dtype is not None:
        base = replace(base, noise_dtype=args.noise_dtype, noise_table_len=args.table_len if args.noise_dtype >= 4 else 0)
    if args.hidden_act == "relu":
        base = replace(base, name=base.name + "-relu", hidden_act=1)
    if args.algorithm == "ars":
        base = replace(base, name=base.name + "-ars", algorithm=1, num_elites=max(1, base.pop // 8), lr=0.02, sigma=0.03)
    elif args.algorithm == "vanilla":
        base = replace(base, name=base.name + "-vanilla", algorithm=2, num_elites=max(1, base.pop // 8), antithetic=0)
    if args.no_antithetic:
        base = replace(base, name=base.name + "-noanti", antithetic=0)
    if args.env_f32:
        base = replace(base, name=base.name + "-envf32", env_dtype=1)
    if args.num_hidden != 2:
        base = replace(base, name=base.name + f"-m{args.num_hidden}", num_hidden=args.num_hidden)
    if args.episodes_per_env != 1:
        base = replace(base, name=base.name + f"-k{args.episodes_per_env}", episodes=args.episodes_per_env)
    w = base if args.done_rule else base.fixed_length()
    a_mat, b_mat, theta = make_inputs(w)

    obs_stats = None
    if args.obs_norm:
        rng = np.random.default_rng([base.seed, 77])
        obs_stats = ((rng.standard_normal(base.obs) * 0.05).astype(np.float32),
                     (1.0 / (0.33 + rng.random(base.obs) * 0.67)).astype(np.float32))

    def setup(wl):
        ctx = EsContext(wl)
        d = ctx.param_count
        dev = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
        if obs_stats is not None:
            ctx.set_obs_norm(dev(obs_stats[0]), dev(obs_stats[1]))
        noise = ctx.alloc_noise()
        if ctx.noise_table:
            ctx.build_noise_table(noise)          # once, outside the timed region (the table does not depend on the generation)
        bufs = dict(noise=noise, ws=ctx.alloc_workspace(), theta=dev(theta), A=dev(a_mat), B=dev(b_mat),
                    m=torch.zeros(d, device="cuda"), v=torch.zeros(d, device="cuda"),
                    ret=torch.empty((wl.pop, ctx.episodes), device="cuda"),
                    len=torch.empty((wl.pop, ctx.episodes), dtype=torch.int32, device="cuda"),
                    fit=torch.empty(wl.pop, device="cuda"), rank=torch.empty(wl.pop, dtype=torch.int32, device="cuda"),
                    shaped=torch.empty(wl.pop, device="cuda"))
        return ctx, bufs

    ctx, bufs = setup(w)
    wall, stage, live = run_generations(torch, ctx, w, bufs, args.steps, args.warmup)
    mean = lambda xs: float(sum(xs) / len(xs))
    median = lambda xs: float(sorted(xs)[len(xs) // 2]) if len(xs) % 2 else float(sum(sorted(xs)[len(xs) // 2 - 1:len(xs) // 2 + 1]) / 2)
    ms_per_step = wall * 1e3 / args.steps
    nominal = w.env_steps
    executed = live if args.done_rule else nominal     # fixed-length: every step of every episode runs
    if not args.done_rule:
        assert live == nominal, f"fixed-length run executed {live} of {nominal} env-steps"
    value = executed * args.steps / wall

    roll_ms = mean(stage["rollout"])
    upd_ms = mean(stage["update"])
    flops = flop_per_env_step(w) * executed
    bf16 = w.dtype == 1
    f32_mfma = (not bf16) and "mfma" in ctx.rollout_kernel        # binary32 on the matrix cores: priced against the fp32 MFMA peak
    peak = MFMA_BF16_PEAK_TFLOPS if bf16 else FP32_VALU_PEAK_TFLOPS
    ach = flops / (roll_ms * 1e-3) / 1e12
    roofline = {"kernel": ctx.rollout_kernel, "bound": "mfma" if (bf16 or f32_mfma) else "alu", "achieved": ach, "peak": peak,
                "unit": "TFLOP/s", "frac": ach / peak, "traffic": None,
                "flop_per_launch": flops, "avg_launch_ms": roll_ms}
    if "mfma" in ctx.rollout_kernel:
        # the environment copies are the 16 columns of the matrix-core tile: with fewer episodes per individual only
        # that share of every MFMA is algorithmic work, whatever the kernel does
        # (the four-copy binary32 kernel uses the 4x4x1 shape: four columns per pass)
        width = 4 if "copies4" in ctx.rollout_kernel else 16
        passes = (ctx.episodes + width - 1) // width
        share = ctx.episodes / (width * passes)
        roofline["column_ceiling"] = share
        roofline["frac_of_column_ceiling"] = (ach / peak) / share
        roofline["columns_per_pass"] = width
    plain = (args.noise_dtype is None and args.algorithm == "openes" and args.hidden_act == "tanh" and not args.obs_norm
             and args.episodes_per_env == 1 and args.num_hidden == 2 and not args.paper_base and args.pop is None
             and not args.no_antithetic and not args.env_f32)
    traffic = (measured_traffic(w.name) if plain else None) or {}
    roofline["traffic"] = traffic.get("rollout_bytes_per_launch")
    if traffic:
        roofline["traffic_source"] = f"profiles/hbm_traffic_{w.name.replace('-', '_')}.txt: two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE) of this command, scaled by a plain copy"
    ub = update_bytes(w, ctx)
    ugbs = ub / (upd_ms * 1e-3) / 1e9
    roofline_update = {"kernel": ctx.update_kernel, "bound": "hbm", "achieved": ugbs, "peak": HBM_PEAK_GBS,
                       "unit": "GB/s", "frac": ugbs / HBM_PEAK_GBS, "traffic": traffic.get("update_bytes_per_launch"),
                       "bytes_per_launch": ub,
                       "avg_launch_ms": upd_ms}
    if w.noise_dtype in (2, 3):      # no noise matrix: the update recomputes every value and is bound by the vector ALUs
        ops = w.noise_rows * ((w.n_params + 3) // 4) * REGEN_VALU_OPS_PER_BLOCK
        tops = ops / (upd_ms * 1e-3) / 1e12
        roofline_update = {"kernel": ctx.update_kernel, "bound": "alu", "achieved": tops, "peak": VALU_PEAK_TLANEOPS,
                           "unit": "T lane-op/s", "frac": tops / VALU_PEAK_TLANEOPS, "traffic": None,
                           "lane_ops_per_launch": ops, "noise_bytes_in_hbm": 0, "avg_launch_ms": upd_ms}

    out = {
        "metric": "env-steps/sec (policy fwd + env step), whole %s generation" % {"openes": "OpenES", "ars": "ARS", "vanilla": "VanillaES"}[args.algorithm],
        "value": value, "unit": "env-steps/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if bf16 else "f32", "data": "synthetic",
        "config": {"workload": f"{base.name}: pop {w.pop} x {w.envs} envs{'' if w.episodes == 1 else ' x %d episodes each' % w.episodes}, T={w.horizon}, MLP {w.obs}-{'-'.join([str(w.hid)] * w.num_hidden)}-{w.act} {args.hidden_act}, "
                               f"{'bf16 operands / fp32 accumulate' if bf16 else 'fp32'}, "
                               f"{'termination rule on (live env-steps counted)' if args.done_rule else 'fixed-length episodes (paper Sec. 5.1 protocol)'}",
                   "population": w.pop, "envs_per_individual": w.envs, "episodes_per_env": w.episodes, "horizon": w.horizon, "params": w.n_params,
                   "noise": {0: "binary32 matrix", 1: "bf16 matrix", 2: "regenerated (binary32 values), no matrix",
                             3: "regenerated (bf16-rounded values), no matrix",
                             4: "rows of a shared binary32 table of %d entries" % w.noise_table_len,
                             5: "rows of a shared bf16 table of %d entries" % w.noise_table_len}[w.noise_dtype],
                   "obs_norm": bool(args.obs_norm), "rollout_kernel": ctx.rollout_kernel},
        "generations_per_s": args.steps / wall,
        "env_steps_per_generation": executed,
        "stage_ms": {k: mean(v) for k, v in stage.items()},
        "stage_ms_median": {k: median(v) for k, v in stage.items()},
        "roofline": roofline,
        "roofline_update": roofline_update,
    }

    if not args.done_rule and not args.no_second_variant:
        ctx2, bufs2 = setup(base)
        wall2, stage2, live2 = run_generations(torch, ctx2, base, bufs2, args.steps, args.warmup)
        out["with_termination_rule"] = {"live_env_steps_per_generation": live2, "ms_per_step": wall2 * 1e3 / args.steps,
                                        "live_env_steps_per_s": live2 * args.steps / wall2,
                                        "generations_per_s": args.steps / wall2,
                                        "stage_ms": {k: mean(v) for k, v in stage2.items()}}
        del ctx2, bufs2
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, obs_norm=obs_stats, full=args.cpu_full)
        out["cpu_baseline"]["host_cpus_visible"] = os.cpu_count()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
