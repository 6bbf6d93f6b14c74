#!/usr/bin/env python3
"""Benchmark of the fused communication + GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg4|cfg5|cfg1]

A step is one pass of the whole path for the workload: for cfg2 (the default, the
configuration the headline metric is quoted on) one ditron_ag_gemm call with the emulated
producer delivering the eight shards in ring order while the GEMM consumes them.  Inputs
are synthetic (seeded generators in synth/), resident in HBM before the timed region.
Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP8_TFLOPS = 5000.0
PEAK_HBM_GBS = 8000.0

# HBM bytes per launch measured with rocprofv3 --pmc (see profiles/), or None if not measured
MEASURED_TRAFFIC = {}


def _cpu_baseline_ag(cfg, shards, b):
    """The oracle, as it stands, on the host cores: the whole cfg2 product in fp64."""
    from oracle import ag_gemm as oag
    t0 = time.perf_counter()
    rows = np.arange(cfg.m)
    oag.ag_gemm(shards, b, rows=rows)
    dt = time.perf_counter() - t0
    flops = 2.0 * cfg.m * cfg.n * cfg.k
    return {"value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())),
            "kind": "oracle", "seconds": dt,
            "sample": f"all {cfg.m} rows x {cfg.n} columns of the workload (numpy fp64 GEMM on decoded inputs)"}


def bench_ag_gemm(args, cfg_id):
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, nk, AgGemmRun

    cfg = synth.CONFIGS[cfg_id]
    shards, b = synth.ag_gemm_inputs(cfg)
    sh = [to_dev(s) for s in shards]
    bd = to_dev(nk(b))
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    flops = 2.0 * cfg.m * cfg.n * cfg.k

    def step():
        st = run(sh, bd, cfg.rank)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        step()
        ev[i][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported a signal time-out")
    kernel_ms = sum(a.elapsed_time(b_) for a, b_ in ev) / args.steps
    ms_per_step = wall * 1e3 / args.steps

    # the same kernel with every shard already in place (flags preset): the GEMM alone
    for _ in range(3):
        run.signals[:cfg.world] = run.epoch + 1
        run(None, bd, cfg.rank, flags=B.EXTERNAL_PRODUCER)
    torch.cuda.synchronize()
    pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.steps):
        run.signals[:cfg.world] = run.epoch + 1
        pe[i][0].record()
        run(None, bd, cfg.rank, flags=B.EXTERNAL_PRODUCER)
        pe[i][1].record()
    torch.cuda.synchronize()
    preset_ms = sum(a.elapsed_time(b_) for a, b_ in pe) / args.steps

    achieved = flops / (kernel_ms * 1e-3) / 1e12
    out = {
        "metric": "TFLOP/s of one rank's AllGather-GEMM share (emulated producer, ring-order arrival)",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg{cfg_id}: AG-GEMM world={cfg.world} rank={cfg.rank} A {cfg.world}x[{cfg.m_per_rank},{cfg.k}] "
                               f"B [{cfg.k},{cfg.n}] stored [n,k] -> C [{cfg.m},{cfg.n}] bf16, fp32 accumulate",
                   "latency_us": kernel_ms * 1e3},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": MEASURED_TRAFFIC.get(f"cfg{cfg_id}"),
                     "kernel": "ag_gemm_kernel (producer work-groups + GEMM tiles in one launch)",
                     "kernel_ms": kernel_ms},
        "gemm_only": {"ms": preset_ms, "achieved": flops / (preset_ms * 1e-3) / 1e12,
                      "frac": flops / (preset_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                      "note": "same kernel, all shards resident and flags preset"},
    }
    if not args.no_cpu:
        out["cpu_baseline"] = _cpu_baseline_ag(cfg, shards, b)
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.workload in ("cfg1", "cfg2"):
        out = bench_ag_gemm(args, int(args.workload[3:]))
    else:
        print(f"bench.py: unknown workload {args.workload}", file=sys.stderr)
        sys.exit(2)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
