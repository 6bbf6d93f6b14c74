#!/usr/bin/env python3
"""Benchmark of the fused communication + GEMM hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2|cfg3|cfg4|cfg5|cfg1|gemm_ar|sweep|moe_sweep|yardstick]

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

# Bytes per launch of the dominant kernel between the L2s and memory, from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE; KiB per dispatch) of the commands given in the profile named with each
# entry, each scaled by what the same counter reads for this script's 256 MiB calibration copy
# (FETCH_SIZE reports 0.500 of the bytes read, WRITE_SIZE 1.000 of the bytes written).  Reads include
# those served by the memory-side cache.  A run cannot collect these itself (the counters need the
# profiler), so every entry says which build it was measured on; re-measure after changing the kernel.
MEASURED_TRAFFIC = {
    # workload: (bytes read + bytes written, profile, kernels as of commit)
    "cfg2": (873.0e6 + 193.0e6, "profiles/ag_gemm_kernel_cfg2.md", "6445342"),   # fused launch; GEMM-only launch 739.8e6 + 58.8e6; algorithmic 251.7e6 (+ 268.4e6 emulated gather)
    "cfg3": (822.4e6 + 251.8e6, "profiles/gemm_rs_kernel_reduce_slots_kernel_cfg3.md", "6a80893"),   # gemm_rs_kernel fused; reduce_slots_kernel 134.3e6 + 16.8e6 = its algorithmic 151.0e6
    "cfg4": (144.8e6 + 6.2e6, "profiles/moe_kernels_cfg4.md", "04f4682"),   # moe_grouped_gemm_kernel (algorithmic 123.2e6); the gather in the routing launch: 67.4e6 + 67.2e6
    "gemm_ar": (1956.3e6 + 269.8e6, "profiles/gemm_ar_kernel_table_shape3.md", "6a80893"),   # fused launch: operand panels ~0.9e9 + eight partials 1.07e9 read; partial + output written
    "moe_rs": (33.1e6 + 67.7e6 + 97.1e6 + 62.9e6 + 33.6e6 + 4.2e6 + 0.1e6, "profiles/moe_rs_kernels_table_shape.md", "04f4682"),   # grouped GEMM + combine (with the peers' copies) + reduction + preparation
    "cfg5": (102.1e6 + 28.5e6, "profiles/ag_gemm_splitk_kernel_cfg5.md", "431892f"),   # ag_gemm_splitk_kernel (fp8) with emulated peers: B 67.1e6 + A + three quarters of the partial tiles out and back; algorithmic 70.3e6
}


def _traffic(key):
    t = MEASURED_TRAFFIC.get(key)
    return None if t is None else t[0]


def _traffic_source(key):
    t = MEASURED_TRAFFIC.get(key)
    return None if t is None else {"profile": t[1], "kernels_as_of_commit": t[2]}


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


class _Rotating:
    """The weight operand of a step, rotating through `copies` device copies of the same values: layers follow
    each other with different weights, so a call does not find its B in the caches (a single copy would stay in
    the 256 MB memory-side cache from step to step)."""

    def __init__(self, tensor, copies):
        self.items = [tensor] + [tensor.clone() for _ in range(max(1, copies) - 1)]
        self.i = 0

    def next(self):
        self.i += 1
        return self.items[self.i % len(self.items)]


def bench_ag_gemm(args, cfg_id):
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, nk, AgGemmRun

    cfg = synth.CONFIGS[cfg_id]
    shards, b = synth.ag_gemm_inputs(cfg)
    sh = [to_dev(s) for s in shards]
    bd = to_dev(nk(b))
    weights = _Rotating(bd, args.weight_copies)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k)
    flops = 2.0 * cfg.m * cfg.n * cfg.k

    def step():
        st = run(sh, weights.next(), cfg.rank)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    _ramp(torch, step)
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
        run(None, weights.next(), cfg.rank, flags=B.FLAGS_PRESET)
    torch.cuda.synchronize()
    pe = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for i in range(args.steps):
        pe[i][0].record()
        run(None, weights.next(), cfg.rank, flags=B.FLAGS_PRESET)
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
                   "weight_copies": args.weight_copies,
                   "latency_us": kernel_ms * 1e3, "latency_us_quantiles": _quantiles_us(ev)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": _traffic(f"cfg{cfg_id}"), "traffic_source": _traffic_source(f"cfg{cfg_id}"),
                     "kernel": "ag_gemm_kernel (producer work-groups + GEMM tiles in one launch)",
                     "kernel_ms": kernel_ms},
        "gemm_only": {"ms": preset_ms, "us_quantiles": _quantiles_us(pe), "achieved": flops / (preset_ms * 1e-3) / 1e12,
                      "frac": flops / (preset_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                      "note": "same kernel, all shards resident and flags preset"},
    }
    st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k)
    stamps = torch.zeros(4 * tc["ntiles"] * tc["splits"], dtype=torch.int32, device="cuda")
    run.epoch += 1
    st = B.ag_gemm(sh, bd, B.B_NK, run.c, None, None, run.ws_raw, run.signals, run.status, stamps, None, cfg.m_per_rank, cfg.n,
                   cfg.k, cfg.world, cfg.rank, B.BF16, run.epoch, B.EMULATE_PRODUCER | B.DUMP_TIMING)
    torch.cuda.synchronize()
    if st == B.OK:
        out["flag_wait"] = _wait_share(torch, B, stamps)
    gather_bytes = 2.0 * cfg.m * cfg.k * 2
    if kernel_ms > preset_ms:
        gbs = gather_bytes / ((kernel_ms - preset_ms) * 1e-3) / 1e9
        out["gather"] = {"bound": "hbm", "bytes": gather_bytes, "us": (kernel_ms - preset_ms) * 1e3, "achieved": gbs,
                         "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                         "note": "the emulated all-gather (read + write of the eight shards by the producer work-groups of the "
                                 "same launch): its bytes over the time it adds to the launch (fused minus flags preset)"}
    if not args.no_cpu:
        out["cpu_baseline"] = _cpu_baseline_ag(cfg, shards, b)
    return out


def _calibration_copy(torch):
    """A plain device-to-device copy of known size, outside every timed region: rocprofv3 --pmc runs of this
    script read FETCH_SIZE / WRITE_SIZE for it, which gives the factor the same counters are scaled by."""
    nbytes = 256 << 20
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    dst.copy_(src)
    torch.cuda.synchronize()
    # the same copy a few more times gives the bandwidth a plain copy reaches on this machine (read + write)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(10)]
    for a, b in ev:
        a.record()
        dst.copy_(src)
        b.record()
    torch.cuda.synchronize()
    best_ms = min(a.elapsed_time(b) for a, b in ev)
    return nbytes, 2.0 * nbytes / (best_ms * 1e-3) / 1e9


def _events(torch, n):
    return [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]


RAMP_SECONDS = 0.3
LAST_QUANTILES = None   # per-step event times of the last _timed() region


def _ramp(torch, step):
    """The chip needs about 0.1 s of sustained load before its clocks settle (measured: the fused cfg 2
    step goes from 0.49 ms to 0.45 ms over the first ~200 launches), so a fixed, untimed ramp precedes
    the W warm-up steps whatever W is."""
    t_ramp = time.perf_counter()
    while time.perf_counter() - t_ramp < RAMP_SECONDS:
        for _ in range(20):
            step()
        torch.cuda.synchronize()


def _events_us(torch, fn, n=100, warm=10):
    """Quantiles (us) of n calls of fn, events around each."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    ev = _events(torch, n)
    for a, b in ev:
        a.record()
        fn()
        b.record()
    torch.cuda.synchronize()
    return _quantiles_us(ev)


def _wait_share(torch, B, records):
    """From the time stamps a DITRON_DUMP_TIMING call wrote (start, wait entered, wait left, end per GEMM
    work-group, 100 MHz ticks): the share of the work-groups' time spent waiting for shard flags."""
    r = records.cpu().numpy().reshape(-1, 4).astype("int64")
    r = r[(r[:, 3] != 0) & (r[:, 0] != 0)]
    if not len(r):
        return None
    wait = (r[:, 2] - r[:, 1]) % (1 << 31)
    busy = (r[:, 3] - r[:, 0]) % (1 << 31)
    span = (r[:, 3].max() - r[:, 0].min()) % (1 << 31)
    return {"work_groups": int(len(r)), "wait_share": float(wait.sum() / busy.sum()), "mean_wait_us": float(wait.mean() / 100.0),
            "mean_work_group_us": float(busy.mean() / 100.0), "first_start_to_last_end_us": float(span / 100.0),
            "note": "in-kernel time stamps of one launch with emulated peers: time between entering and leaving the shard-flag wait over "
                    "the work-group's lifetime, summed over the GEMM work-groups"}


def _quantiles_us(ev):
    t = sorted(a.elapsed_time(b) * 1e3 for a, b in ev)
    pick = lambda q: t[min(len(t) - 1, int(q * len(t)))]
    return {"median": pick(0.5), "p10": pick(0.1), "p90": pick(0.9)}


def _timed(torch, args, step):
    """W warm-up steps, then K timed steps with events around each; returns (ms per step by the
    host clock around the whole region, mean ms between the per-step events)."""
    _ramp(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev = _events(torch, args.steps)
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        step()
        ev[i][1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    global LAST_QUANTILES
    LAST_QUANTILES = _quantiles_us(ev)
    return wall * 1e3 / args.steps, sum(a.elapsed_time(b) for a, b in ev) / args.steps


def bench_gemm_rs(args):
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, nk, GemmRsRun

    cfg = synth.CONFIGS[3]
    d, m_r = cfg.rank, cfg.m_per_rank
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    run = GemmRsRun(B, cfg.world, cfg.m, cfg.n, cfg.k, chunks=4)
    zero = torch.zeros((m_r, cfg.n), dtype=torch.int16, device="cuda")
    # the blocks the peers would send: their own partial products' rows for this rank
    peers = []
    for s in range(cfg.world):
        if s == d:
            peers.append(zero)
            continue
        st = run(to_dev(a_list[s]), to_dev(nk(b_list[s])), [zero] * cfg.world, s)
        assert st == B.OK
        torch.cuda.synchronize()
        peers.append(run.gemm_out[d * m_r:(d + 1) * m_r].clone())
    ad, bd = to_dev(a_list[d]), to_dev(nk(b_list[d]))
    weights = _Rotating(bd, args.weight_copies)

    def step():
        st = run(ad, weights.next(), peers, d)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    ms_per_step, ev_ms = _timed(torch, args, step)
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported a signal time-out")
    flops = 2.0 * cfg.m * cfg.n * cfg.k

    # the same call with the peers' blocks already in the scatter buffer and their flags preset: the GEMM
    # kernel without the emulated-peer work-groups, then the gated reduction
    for _ in range(3):
        run(ad, weights.next(), None, d, flags=B.FLAGS_PRESET)
    torch.cuda.synchronize()
    pe = _events(torch, args.steps)
    for i in range(args.steps):
        pe[i][0].record()
        run(ad, weights.next(), None, d, flags=B.FLAGS_PRESET)
        pe[i][1].record()
    torch.cuda.synchronize()
    preset_ms = sum(a.elapsed_time(b) for a, b in pe) / args.steps

    # the reduction alone on buffer sets that rotate through more than the 256 MB last-level cache
    nsets = 4
    sets = [[torch.randint(-30000, 30000, (m_r, cfg.n), dtype=torch.int16, device="cuda") for _ in range(cfg.world)]
            for _ in range(nsets)]
    outs = [torch.empty((m_r, cfg.n), dtype=torch.int16, device="cuda") for _ in range(nsets)]
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    for i in range(2 * nsets):
        B.reduce_slots(sets[i % nsets], outs[i % nsets], None, status, m_r, cfg.n, cfg.world, 1, 1)
    torch.cuda.synchronize()
    nrep = 40
    ev = _events(torch, nrep)
    for i in range(nrep):
        ev[i][0].record()
        B.reduce_slots(sets[i % nsets], outs[i % nsets], None, status, m_r, cfg.n, cfg.world, 1, 1)
        ev[i][1].record()
    torch.cuda.synchronize()
    red_ms = sum(a.elapsed_time(b) for a, b in ev) / nrep
    red_bytes = (cfg.world + 1) * m_r * cfg.n * 2
    red_gbs = red_bytes / (red_ms * 1e-3) / 1e9

    achieved = flops / (ev_ms * 1e-3) / 1e12
    out = {
        "metric": "TFLOP/s of one rank's GEMM-ReduceScatter share (GEMM + emulated peer arrival + reduction)",
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg3: GEMM-RS world={cfg.world} rank={d} A [{cfg.m},{cfg.k}] B [{cfg.k},{cfg.n}] stored [n,k], "
                               f"7 peer blocks [{m_r},{cfg.n}] bf16, 4 row chunks per block", "weight_copies": args.weight_copies,
                   "latency_us": ev_ms * 1e3},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": _traffic("cfg3"), "traffic_source": _traffic_source("cfg3"),
                     "kernel": "gemm_rs_kernel + reduce_slots_kernel (whole step between events)", "kernel_ms": ev_ms},
        "flags_preset": {"ms": preset_ms, "us_quantiles": _quantiles_us(pe), "achieved": flops / (preset_ms * 1e-3) / 1e12,
                         "frac": flops / (preset_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
                         "note": "same entry point, peer blocks resident and arrival flags preset: gemm_rs_kernel without "
                                 "emulated-peer work-groups + the gated reduce_slots_kernel"},
        "reduction": {"bound": "hbm", "achieved": red_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                      "frac": red_gbs / PEAK_HBM_GBS, "us": red_ms * 1e3, "bytes": red_bytes,
                      "note": "reduce_slots_kernel alone, 4 rotating buffer sets (604 MB) so the 256 MB cache cannot hold them"},
    }
    if not args.no_cpu:
        from oracle import gemm_rs as ors
        t0 = time.perf_counter()
        ors.gemm_rs(a_list, b_list, d)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": flops / dt / 1e12, "unit": "TFLOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())), "kind": "oracle",
                               "seconds": dt, "sample": "the rank's whole output block (sum over 8 ranks of [1024,3584].[3584,8192] in fp64)"}
    return out


def bench_gemm_ar(args):
    """GEMM + AllReduce (one-shot) at shape 3 of the paper's GEMM + AllReduce table under tensor parallel 8:
    M 8192, N 8192, K 28672 / 8 (the operands of cfg3), the seven peers' partials resident in HBM."""
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, nk, GemmArRun

    cfg = synth.CONFIGS[3]
    d = cfg.rank
    a_list, b_list = synth.gemm_rs_inputs(cfg)
    solo = GemmArRun(B, 1, cfg.m, cfg.n, cfg.k)
    peers = []
    for s in range(cfg.world):          # the peers' published partials, made by the same GEMM
        if s == d:
            peers.append(None)
            continue
        st = solo(to_dev(a_list[s]), to_dev(nk(b_list[s])), None, 0)
        assert st == B.OK
        torch.cuda.synchronize()
        peers.append(solo.gemm_out.clone())
    ad, bd = to_dev(a_list[d]), to_dev(nk(b_list[d]))
    run = GemmArRun(B, cfg.world, cfg.m, cfg.n, cfg.k)

    weights = _Rotating(bd, args.weight_copies)

    def step():
        st = run(ad, weights.next(), peers, d)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    ms_per_step, ev_ms = _timed(torch, args, step)
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported a signal time-out")
    flops = 2.0 * cfg.m * cfg.n * cfg.k
    red_bytes = (cfg.world + 1) * cfg.m * cfg.n * 2

    # the GEMM with its per-tile flags alone (world 1: the consumer only copies the partial)
    for _ in range(5):
        solo(ad, bd, None, 0)
    torch.cuda.synchronize()
    ev = _events(torch, args.steps)
    for i in range(args.steps):
        ev[i][0].record()
        solo(ad, bd, None, 0)
        ev[i][1].record()
    torch.cuda.synchronize()
    solo_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps

    # the two-shot form of the same problem: this rank reduces the tiles it owns and stores them into eight output
    # buffers; the tiles the seven peers own are copied into its output from what they broadcast
    outs = [run.out if s == d else torch.empty((cfg.m, cfg.n), dtype=torch.int16, device="cuda") for s in range(cfg.world)]
    reduced = [None if s == d else peers[s] for s in range(cfg.world)]   # any resident [m, n] buffers: the values do not matter for time

    def two_shot():
        run.epoch += 1
        st = B.gemm_ar_two_shot(ad, bd, B.B_NK, run.gemm_out, peers, outs, reduced, run.signals, run.status, None,
                                cfg.m, cfg.n, cfg.k, cfg.world, d, run.epoch, B.EMULATE_PRODUCER)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    for _ in range(5):
        two_shot()
    torch.cuda.synchronize()
    ev = _events(torch, args.steps)
    for i in range(args.steps):
        ev[i][0].record()
        two_shot()
        ev[i][1].record()
    torch.cuda.synchronize()
    two_ms = sum(a.elapsed_time(b) for a, b in ev) / args.steps
    ev2 = ev
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported a signal time-out")
    del outs

    # the all-reduce of the eight partials alone, as a plain streaming kernel over the whole chip
    slots = [run.gemm_out if s == d else peers[s] for s in range(cfg.world)]
    status = torch.zeros(B.STATUS_WORDS, dtype=torch.int32, device="cuda")
    for _ in range(3):
        B.reduce_slots(slots, run.out, None, status, cfg.m, cfg.n, cfg.world, 1, 1)
    torch.cuda.synchronize()
    ev = _events(torch, 20)
    for i in range(20):
        ev[i][0].record()
        B.reduce_slots(slots, run.out, None, status, cfg.m, cfg.n, cfg.world, 1, 1)
        ev[i][1].record()
    torch.cuda.synchronize()
    red_ms = sum(a.elapsed_time(b) for a, b in ev) / 20

    achieved = flops / (ev_ms * 1e-3) / 1e12
    out = {
        "metric": "TFLOP/s of one rank's GEMM + AllReduce share (GEMM with per-tile flags, one-shot software all-reduce)",
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"gemm_ar: GEMM-AR world={cfg.world} rank={d} A [{cfg.m},{cfg.k}] B [{cfg.k},{cfg.n}] stored [n,k], "
                               f"7 peer partials [{cfg.m},{cfg.n}] bf16 resident -> out [{cfg.m},{cfg.n}] bf16", "weight_copies": args.weight_copies,
                   "latency_us": ev_ms * 1e3},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": _traffic("gemm_ar"), "traffic_source": _traffic_source("gemm_ar"),
                     "kernel": "gemm_ar_kernel (GEMM tiles + all-reduce consumers in one launch)", "kernel_ms": ev_ms},
        "two_shot": {"ms": two_ms, "achieved": flops / (two_ms * 1e-3) / 1e12, "us_quantiles": _quantiles_us(ev2),
                     "note": "ditron_gemm_ar_two_shot on the same operands: 1/8 of the tiles reduced here and stored to eight outputs, "
                             "7/8 copied in from the emulated peers' broadcasts"},
        "gemm_and_copy": {"ms": solo_ms, "note": "world 1: the GEMM with its tile flags; the consumer only copies the partial (268 MB)"},
        "allreduce_alone": {"bound": "hbm", "bytes": red_bytes, "ms": red_ms, "achieved": red_bytes / (red_ms * 1e-3) / 1e9,
                            "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": red_bytes / (red_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                            "note": "reduce_slots_kernel over the same eight [8192,8192] partials: what the all-reduce costs when "
                                    "nothing overlaps it (the whole chip streaming)"},
    }
    if not args.no_cpu:
        from oracle import gemm_ar as oar
        rows = np.arange(0, cfg.m, 8)
        t0 = time.perf_counter()
        oar.gemm_ar(a_list, b_list, rows=rows)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": 2.0 * len(rows) * cfg.n * cfg.k * cfg.world / dt / 1e12, "unit": "TFLOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())), "kind": "oracle", "seconds": dt,
                               "sample": f"every 8th row of the output ({len(rows)} rows x {cfg.n} columns, all 8 ranks' products in fp64; "
                                         "the oracle computes every rank's share, the GPU figure counts one)"}
    return out


def bench_moe(args):
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, MoeRun

    cfg = synth.CONFIGS[4]
    xs, ids, w = synth.moe_inputs(cfg)
    e0 = cfg.rank * cfg.num_local_experts
    max_rows = 4096
    run = MoeRun(B, cfg.world, cfg.tokens_per_rank, cfg.k, cfg.n, cfg.num_experts, cfg.top_k, cfg.num_local_experts, max_rows)
    xd = [to_dev(x) for x in xs]
    idd = to_dev(ids)
    # the expert weights (101 MB) rotate through three copies, so that they stream from HBM and not from the
    # 256 MB memory-side cache
    nsets = 3
    wds = [to_dev(np.ascontiguousarray(np.transpose(w, (0, 2, 1)))) for _ in range(nsets)]
    it = [0]

    def step():
        it[0] += 1
        st = run(xd, idd, wds[it[0] % nsets], e0, cfg.rank)
        if st != B.OK:
            raise RuntimeError(B.status_string(st))

    ms_per_step, ev_ms = _timed(torch, args, step)
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported an error")
    R = int(run.offsets.cpu()[-1])
    # the gather on its own: the same call with a routing that sends nothing to the local experts, so the grouped
    # GEMM launch has no tile and the step is the routing launch (routing scan beside the emulated all-gather)
    nowhere = torch.full_like(idd, (e0 + cfg.num_local_experts) % cfg.num_experts)
    gather_us = _events_us(torch, lambda: run(xd, nowhere, wds[0], e0, cfg.rank))["median"]
    gather_bytes = 2.0 * cfg.world * cfg.tokens_per_rank * cfg.k * 2
    step()          # leave the buffers as the timed steps had them
    torch.cuda.synchronize()
    flops = 2.0 * R * cfg.k * cfg.n
    w_bytes = w.size * 2
    alg_bytes = w_bytes + R * cfg.k * 2 + R * cfg.n * 2
    gbs = alg_bytes / (ev_ms * 1e-3) / 1e9
    out = {
        "metric": "TFLOP/s of one rank's MoE AllGather + grouped GEMM share (route + schedule + gather + GEMM)",
        "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"cfg4: MoE world={cfg.world} rank={cfg.rank} tokens 8x{cfg.tokens_per_rank} hidden {cfg.k} inter {cfg.n} "
                               f"{cfg.num_experts} experts top-{cfg.top_k}, {cfg.num_local_experts} local, R={R}", "latency_us": ev_ms * 1e3},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                     "traffic": _traffic("cfg4"), "traffic_source": _traffic_source("cfg4"),
                     "kernel": "moe_route_kernel + moe_grouped_gemm_kernel (whole step between events)", "kernel_ms": ev_ms,
                     "bytes": alg_bytes},
        "gather": {"bound": "hbm", "bytes": gather_bytes, "us": gather_us, "achieved": gather_bytes / gather_us / 1e3,
                   "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gather_bytes / gather_us / 1e3 / PEAK_HBM_GBS,
                   "note": "the emulated all-gather of the token shards (read + write) beside the routing scan: the call with a "
                           "routing that sends nothing to the local experts, events around it (includes the launch of both kernels)"},
    }
    if not args.no_cpu:
        from oracle import moe as omoe
        t0 = time.perf_counter()
        omoe.grouped_gemm(xs, ids, w, cfg.world, cfg.num_experts, e0)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": flops / dt / 1e12, "unit": "TFLOP/s",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())), "kind": "oracle",
                               "seconds": dt, "sample": "the whole workload (route in Python loops + fp64 grouped GEMM)"}
    return out


# Per-rank shares (world 8) of the paper's evaluation shapes: Appendix "Evaluation Setup", tables
# "Shapes for AllGather+GEMM" (N divided by the ranks) and "Shapes for GEMM+ReduceScatter" (K divided).
SWEEP_AG = [("LLaMA3-7B", 1376, 4096), ("LLaMA3.1-8B", 1792, 4096), ("LLaMA3.1-70B", 3584, 8192),
            ("LLaMA3.1-405B", 6656, 16384), ("Mistral-7B", 1792, 4096), ("Qwen2-72B", 3696, 8192)]
SWEEP_RS = [("LLaMA3-7B", 4096, 1376), ("LLaMA3.1-8B", 4096, 1792), ("LLaMA3.1-70B", 8192, 3584),
            ("LLaMA3.1-405B", 16384, 6656), ("Mistral-7B", 4096, 1792), ("Qwen2-72B", 8192, 3696)]


def bench_sweep(args):
    """Both bf16 operators over the shapes of the paper's two dense tables (M = 8192, world 8, rank 0),
    random N(0,1) / N(0,1/K) bf16 generated on the device.  One step = all twelve problems once."""
    import math
    import torch
    from paper_2605_02953_amd import binding as B
    from gpu_util import AgGemmRun, GemmRsRun

    world, m_r = 8, 1024
    m = world * m_r

    def rnd(shape, std):
        return (torch.randn(shape, device="cuda") * std).to(torch.bfloat16).view(torch.int16)

    rows, problems = [], []
    for name, n, k in SWEEP_AG:
        run = AgGemmRun(B, world, m_r, n, k)
        sh = [rnd((m_r, k), 1.0) for _ in range(world)]
        bd = rnd((n, k), k ** -0.5)

        def fused(run=run, sh=sh, bd=bd):
            assert run(sh, bd, 0) == B.OK

        def preset(run=run, bd=bd):
            return lambda: run(None, bd, 0, flags=B.FLAGS_PRESET)

        problems.append(("ag_gemm", name, n, k, fused, preset, run))
    for name, n, k in SWEEP_RS:
        run = GemmRsRun(B, world, m, n, k, chunks=4)
        a, bd = rnd((m, k), 1.0), rnd((n, k), k ** -0.5)
        peers = [rnd((m_r, n), 1.0) for _ in range(world)]

        def fused(run=run, a=a, bd=bd, peers=peers):
            assert run(a, bd, peers, 0) == B.OK

        def preset(run=run, a=a, bd=bd):
            return lambda: run(a, bd, None, 0, flags=B.FLAGS_PRESET)

        problems.append(("gemm_rs", name, n, k, fused, preset, run))

    def step():
        for pr in problems:
            pr[4]()

    _ramp(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    reps = max(1, args.steps)
    t0 = time.perf_counter()
    per = [[] for _ in problems]
    for _ in range(reps):
        for i, pr in enumerate(problems):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pr[4]()
            e1.record()
            per[i].append((e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    pre = [[] for _ in problems]
    for _ in range(reps):
        for i, pr in enumerate(problems):
            call = pr[5]()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            st = call()
            e1.record()
            assert st == B.OK
            pre[i].append((e0, e1))
    torch.cuda.synchronize()
    total_flops, logs = 0.0, []
    for i, (op, name, n, k, _, _, run) in enumerate(problems):
        if run.status.cpu().tolist()[0] != 0:
            raise RuntimeError("kernel reported a signal time-out")
        flops = 2.0 * m * n * k
        total_flops += flops
        us = _quantiles_us(per[i])["median"]
        us_p = _quantiles_us(pre[i])["median"]
        rows.append({"op": op, "model": name, "m": m, "n": n, "k": k, "us": us, "tflops": flops / us / 1e6,
                     "us_flags_preset": us_p, "tflops_flags_preset": flops / us_p / 1e6})
        logs.append(math.log(flops / us / 1e6))
    ms_per_step = wall * 1e3 / reps
    geo = math.exp(sum(logs) / len(logs))
    return {
        "metric": "TFLOP/s over one pass of the paper's 6 AG-GEMM and 6 GEMM-RS shapes (per-rank share, world 8)",
        "value": total_flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": reps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "sweep: AG-GEMM [8192, N/8, K] and GEMM-RS [8192, N, K/8] for the six models of the paper's shape tables"},
        "roofline": {"bound": "mfma", "achieved": geo, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": geo / PEAK_BF16_TFLOPS,
                     "traffic": None, "kernel": "geometric mean over the twelve problems (events around each call)"},
        "sweep": rows,
    }


# The paper's AllGather+MoE shapes (Appendix "Evaluation Setup", table "Shapes for AllGather+MoE and
# MoE+AllReduce": tokens 8192) in its tensor-parallel placement: every expert on every rank, the
# intermediate dimension divided by the 8 ranks.  (name, hidden, intermediate / 8, experts, top_k)
SWEEP_MOE = [("Qwen1.5-MoE-A2.7B", 2048, 176, 60, 4), ("Mixtral-8x7B", 14336, 512, 8, 2),
             ("Mixtral-8x22B", 16384, 768, 8, 2), ("DeepSeek-MoE", 1408, 256, 64, 6)]


def bench_moe_rs(args):
    """MoE down-projection + ReduceScatter at the shape of the paper's MoE+RS table (8192 tokens, hidden 2048,
    intermediate 1536 over 8 ranks, 32 experts, top-2), tensor-parallel placement: every expert on the rank, its
    slice of the intermediate size.  Routing tables are made with torch (stable sort by expert); activations and
    weights N(0,1) / N(0,1/intermediate) bf16 made on the device."""
    import torch
    from paper_2605_02953_amd import binding as B

    world, t_r, hidden, inter, experts, top_k, chunks = 8, 1024, 2048, 1536 // 8, 32, 2, 4
    tokens, rows = world * t_r, world * t_r * top_k
    g = torch.Generator(device="cuda").manual_seed(11)
    i32 = dict(dtype=torch.int32, device="cuda")
    ids = torch.rand((tokens, experts), device="cuda", generator=g).argsort(dim=1)[:, :top_k].reshape(-1)
    order = torch.sort(ids, stable=True).indices.to(torch.int32).contiguous()          # gather_idx: assignments grouped by expert
    offsets = torch.zeros(experts + 1, **i32)
    offsets[1:] = torch.bincount(ids, minlength=experts).cumsum(0).to(torch.int32)
    h = torch.randn((rows, inter), device="cuda", generator=g).to(torch.bfloat16).view(torch.int16)
    nsets = 3
    w2 = [(torch.randn((experts, hidden, inter), device="cuda", generator=g) * (inter * world) ** -0.5).to(torch.bfloat16).view(torch.int16)
          for _ in range(nsets)]
    gate = torch.rand((tokens * top_k,), device="cuda", generator=g)
    peers = [None if s == 0 else torch.randn((t_r, hidden), device="cuda", generator=g).to(torch.bfloat16).view(torch.int16) for s in range(world)]
    max_rows = rows
    y = torch.zeros((max_rows, hidden), dtype=torch.int16, device="cuda")
    inv = torch.zeros((tokens * top_k,), **i32)
    rec = torch.zeros((1 + 5 * B.moe_max_tiles(max_rows, experts),), **i32)
    combined = torch.zeros((tokens, hidden), dtype=torch.int16, device="cuda")
    scatter = torch.zeros((world, t_r, hidden), dtype=torch.int16, device="cuda")
    out_t = torch.zeros((t_r, hidden), dtype=torch.int16, device="cuda")
    signals = torch.zeros(B.signal_words(world, chunks), **i32)
    status = torch.zeros(B.STATUS_WORDS, **i32)
    state = {"epoch": 0, "it": 0}

    def make_step(flags):
        def step():
            state["epoch"] += 1
            state["it"] += 1
            st = B.moe_grouped_gemm_rs(h, w2[state["it"] % nsets], B.B_NK, gate, order, offsets, y, inv, rec, combined,
                                       None if flags == B.FLAGS_PRESET else peers, scatter, out_t, signals, status, None, t_r, hidden,
                                       inter, experts, top_k, experts, max_rows, world, 0, chunks, state["epoch"], flags)
            if st != B.OK:
                raise RuntimeError(B.status_string(st))
        return step

    step = make_step(B.EMULATE_PRODUCER)
    ms_per_step, ev_ms = _timed(torch, args, step)
    if status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported an error")
    quant = LAST_QUANTILES
    preset = _events_us(torch, make_step(B.FLAGS_PRESET), n=100, warm=10)
    flops = 2.0 * rows * inter * hidden
    slot = t_r * hidden * 2
    # h and the weights in, y out and back in, the combined block out, the reduction's world slots in and its result out
    alg_bytes = rows * inter * 2 + experts * hidden * inter * 2 + 2 * rows * hidden * 2 + tokens * hidden * 2 + (world + 1) * slot
    peer_bytes = 2.0 * (world - 1) * slot
    gbs = (alg_bytes + peer_bytes) / (ev_ms * 1e-3) / 1e9
    return {
        "metric": "time (us) of one rank's MoE down-projection + ReduceScatter share (emulated peers)",
        "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"moe_rs: grouped GEMM [{rows}, {inter}] x [{experts}, {inter}, {hidden}] + top-{top_k} combine + reduce-scatter over "
                               f"{world} slots of [{t_r}, {hidden}] ({chunks} row chunks): the paper's MoE+RS table shape at tensor parallel 8",
                   "latency_us": ev_ms * 1e3, "latency_us_quantiles": quant, "tflops": flops / (ev_ms * 1e-3) / 1e12},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS, "traffic": _traffic("moe_rs"),
                     "traffic_source": _traffic_source("moe_rs"),
                     "kernel": "moe_rs_prepare_kernel + moe_grouped_gemm_kernel + moe_combine_kernel + reduce_slots_kernel (whole step between events)",
                     "kernel_ms": ev_ms, "bytes": alg_bytes + peer_bytes,
                     "note": "algorithmic bytes of the four launches plus the emulated peers' copies (read + write of 7 blocks)"},
        "flags_preset_us": preset,
    }


def bench_moe_sweep(args):
    """MoE AllGather + grouped GEMM over the four shapes of the paper's MoE table, all experts local
    (expert_begin 0), 8 x 1024 tokens, uniform top-k routing, N(0,1) / N(0,1/hidden) bf16 made on the
    device.  One step = the four problems once."""
    import math
    import torch
    from paper_2605_02953_amd import binding as B
    from gpu_util import MoeRun

    world, t_r = 8, 1024
    g = torch.Generator(device="cuda").manual_seed(7)
    problems = []
    for name, hidden, inter, experts, top_k in SWEEP_MOE:
        rows = world * t_r * top_k
        run = MoeRun(B, world, t_r, hidden, inter, experts, top_k, experts, rows)
        xs = [torch.randn((t_r, hidden), device="cuda", generator=g).to(torch.bfloat16).view(torch.int16) for _ in range(world)]
        # top_k distinct experts per token: the first top_k of a random permutation
        ids = torch.rand((world * t_r, experts), device="cuda", generator=g).argsort(dim=1)[:, :top_k].to(torch.int32).contiguous()
        w = (torch.randn((experts, inter, hidden), device="cuda", generator=g) * hidden ** -0.5).to(torch.bfloat16).view(torch.int16)

        def call(run=run, xs=xs, ids=ids, w=w):
            st = run(xs, ids, w, 0, 0)
            if st != B.OK:
                raise RuntimeError(B.status_string(st))

        # the same call with nothing routed to the one local expert it is given: the gather + routing launch alone
        ids_none = torch.zeros_like(ids)
        run_g = MoeRun(B, world, t_r, hidden, inter, experts, top_k, 1, 1024)

        def gather_only(run_g=run_g, xs=xs, ids_none=ids_none, w=w):
            st = run_g(xs, ids_none, w, 1, 0)
            if st != B.OK:
                raise RuntimeError(B.status_string(st))

        problems.append((name, hidden, inter, experts, top_k, rows, call, run, gather_only))

    def step():
        for pr in problems:
            pr[6]()

    _ramp(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    reps = max(1, args.steps)
    per = [[] for _ in problems]
    t0 = time.perf_counter()
    for _ in range(reps):
        for i, pr in enumerate(problems):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            pr[6]()
            e1.record()
            per[i].append((e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rows_out, total_flops, logs = [], 0.0, []
    for i, (name, hidden, inter, experts, top_k, rows, _, run, gather_only) in enumerate(problems):
        if run.status.cpu().tolist()[0] != 0:
            raise RuntimeError("kernel reported an error")
        g_us = _events_us(torch, gather_only, n=30, warm=5)["median"]
        g_bytes = 2.0 * world * t_r * hidden * 2
        assert int(run.offsets.cpu()[-1]) == rows
        flops = 2.0 * rows * hidden * inter
        total_flops += flops
        us = _quantiles_us(per[i])["median"]
        alg_bytes = experts * inter * hidden * 2 + world * t_r * hidden * 2 + rows * inter * 2
        rows_out.append({"model": name, "tokens": world * t_r, "hidden": hidden, "inter": inter, "experts": experts, "top_k": top_k,
                         "rows": rows, "us": us, "tflops": flops / us / 1e6, "algorithmic_gbs": alg_bytes / us / 1e3,
                         "gather_bytes": g_bytes, "gather_us": g_us, "gather_gbs": g_bytes / g_us / 1e3})
        logs.append(math.log(flops / us / 1e6))
    ms_per_step = wall * 1e3 / reps
    geo = math.exp(sum(logs) / len(logs))
    return {
        "metric": "TFLOP/s over one pass of the paper's 4 AllGather+MoE shapes (tensor-parallel placement, per-rank share, world 8)",
        "value": total_flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": reps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "moe_sweep: route + emulated all-gather + grouped GEMM [tokens*top_k, hidden] x [experts, hidden, inter/8] for the four models of the paper's MoE table"},
        "roofline": {"bound": "mfma", "achieved": geo, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": geo / PEAK_BF16_TFLOPS,
                     "traffic": None, "kernel": "geometric mean over the four problems (events around each call: both launches)"},
        "sweep": rows_out,
    }


def bench_fp8(args):
    import torch
    import synth
    from paper_2605_02953_amd import binding as B
    from gpu_util import to_dev, nk, AgGemmRun

    cfg = synth.CONFIGS[5]
    a, sa, b, sb = synth.fp8_ag_gemm_inputs(cfg)
    ad = [to_dev(x) for x in a]
    # rotate the weight matrix through several copies so it is streamed from HBM, not from cache
    nsets = 5
    bds = [to_dev(nk(b)) for _ in range(nsets)]
    sad, sbd = to_dev(sa), to_dev(sb)
    run = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1, tuning=B.tuning(decode_variant=args.decode_variant))
    it = [0]

    def make_step(r, flags=None):
        # the arguments are marshalled once per weight copy; a step only advances the epoch
        calls = [B.PreparedAgGemm(ad if flags is None else None, bd_, B.B_NK, r.c, sad, sbd, r.ws_raw, r.signals, r.status, None,
                                  None, cfg.m_per_rank, cfg.n, cfg.k, cfg.world, cfg.rank, B.FP8_E4M3,
                                  B.EMULATE_PRODUCER if flags is None else flags, tuning=r.tuning) for bd_ in bds]

        def step():
            it[0] += 1
            r.epoch += 1
            st = calls[it[0] % nsets](r.epoch)
            if st != B.OK:
                raise RuntimeError(B.status_string(st))
        return step

    step = make_step(run)
    ms_per_step, ev_ms = _timed(torch, args, step)
    if run.status.cpu().tolist()[0] != 0:
        raise RuntimeError("kernel reported a signal time-out")
    quant = LAST_QUANTILES
    # the same call with the gathered operand resident (no emulated peers, no waits), and every kernel variant
    # of the decode path, each timed the same way (events around each call, B rotating)
    def events_us(fn, n=200):
        for _ in range(20):
            fn()
        torch.cuda.synchronize()
        ev = _events(torch, n)
        for a_, b_ in ev:
            a_.record()
            fn()
            b_.record()
        torch.cuda.synchronize()
        q = _quantiles_us(ev)
        # 100 calls between one pair of events: launches queue up behind one another, so this is the
        # kernel's own duration plus the gap between two dispatches
        e0, e1 = _events(torch, 1)[0]
        e0.record()
        for _ in range(100):
            fn()
        e1.record()
        torch.cuda.synchronize()
        q["back_to_back"] = e0.elapsed_time(e1) * 10.0
        return q

    preset = events_us(make_step(run, B.FLAGS_PRESET))
    st, tc0 = B.tile_config(0, cfg.m, cfg.n, cfg.k, B.FP8_E4M3, run.tuning)
    stamps = torch.zeros(4 * tc0["ntiles"] * tc0["splits"], dtype=torch.int32, device="cuda")
    run.epoch += 1
    st = B.ag_gemm(ad, bds[0], B.B_NK, run.c, sad, sbd, run.ws_raw, run.signals, run.status, stamps, None, cfg.m_per_rank, cfg.n,
                   cfg.k, cfg.world, cfg.rank, B.FP8_E4M3, run.epoch, B.EMULATE_PRODUCER | B.DUMP_TIMING, tuning=run.tuning)
    torch.cuda.synchronize()
    wait_share = _wait_share(torch, B, stamps) if st == B.OK else None
    # what one tiny launch costs between two events on this machine (the floor of any single-call latency)
    tiny = torch.zeros((1, 8), dtype=torch.int16, device="cuda")
    floor_us = events_us(lambda: B.reduce_slots([tiny], tiny.clone(), None, run.status, 1, 8, 1, 1, 1))
    variants = {}
    names = {1: "128x32 tiles, whole contraction", 2: "128x128 tiles, split contraction", 3: "128x64 tiles, split contraction",
             4: "16-row tiles, one per shard"}
    for v in (1, 2, 3, 4):
        rv = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1, tuning=B.tuning(decode_variant=v))
        st, tc = B.tile_config(0, cfg.m, cfg.n, cfg.k, B.FP8_E4M3, B.tuning(decode_variant=v))
        variants[str(v)] = {"what": names[v], "splits": tc["splits"], "emulated_peers_us": events_us(make_step(rv)),
                            "flags_preset_us": events_us(make_step(rv, B.FLAGS_PRESET))}
        if rv.status.cpu().tolist()[0] != 0:
            raise RuntimeError("kernel reported a signal time-out")
    # the same call recorded once in a HIP graph (the epoch lives in memory and the kernel advances it) and replayed:
    # what a caller that cannot afford the per-call host work sees
    rg = AgGemmRun(B, cfg.world, cfg.m_per_rank, cfg.n, cfg.k, esize=1, tuning=run.tuning)
    gflags = B.EMULATE_PRODUCER | B.EPOCH_IN_MEMORY
    per_graph = 4 * nsets
    for bd_ in bds[:2]:     # the first calls configure the kernel, outside the capture
        B.ag_gemm(ad, bd_, B.B_NK, rg.c, sad, sbd, rg.ws_raw, rg.signals, rg.status, None, None, cfg.m_per_rank, cfg.n, cfg.k,
                  cfg.world, cfg.rank, B.FP8_E4M3, 0, gflags, tuning=rg.tuning)
    torch.cuda.synchronize()
    side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        try:
            for i in range(per_graph):
                st = B.ag_gemm(ad, bds[i % nsets], B.B_NK, rg.c, sad, sbd, rg.ws_raw, rg.signals, rg.status, None, None, cfg.m_per_rank,
                               cfg.n, cfg.k, cfg.world, cfg.rank, B.FP8_E4M3, 0, gflags, side, rg.tuning)
        finally:
            graph.capture_end()
    graph_replay = None
    if st == B.OK:
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        reps = 10
        e0, e1 = _events(torch, 1)[0]
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            graph.replay()
        e1.record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if rg.status.cpu().tolist()[0] != 0:
            raise RuntimeError("kernel reported a signal time-out")
        graph_replay = {"us_per_call": e0.elapsed_time(e1) * 1e3 / (reps * per_graph), "wall_us_per_call": wall * 1e6 / (reps * per_graph),
                        "calls_per_graph": per_graph, "replays": reps,
                        "note": "DITRON_EPOCH_IN_MEMORY: the call recorded once per weight copy in one HIP graph, emulated peers included; "
                                "time of the replays over the calls they hold"}
    flops = 2.0 * cfg.m * cfg.n * cfg.k
    alg_bytes = cfg.k * cfg.n + cfg.m * cfg.k + cfg.m * cfg.n * 2
    gbs = alg_bytes / (ev_ms * 1e-3) / 1e9
    out = {
        "metric": "latency (us) of one rank's decode-shaped fp8 AllGather-GEMM share",
        "value": ms_per_step * 1e3, "unit": "us",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "fp8_e4m3", "data": "synthetic",
        "config": {"workload": f"cfg5: fp8 AG-GEMM world={cfg.world} A 8x[{cfg.m_per_rank},{cfg.k}] B [{cfg.k},{cfg.n}] stored [n,k] "
                               f"-> C [{cfg.m},{cfg.n}] bf16; weights rotated over {nsets} copies", "latency_us": ev_ms * 1e3,
                   "tflops": flops / (ev_ms * 1e-3) / 1e12},
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBS,
                     "traffic": _traffic("cfg5"), "traffic_source": _traffic_source("cfg5"), "kernel": "ag_gemm_splitk_kernel (fp8)", "kernel_ms": ev_ms,
                     "bytes": alg_bytes},
        "flags_preset_us": preset,
        "flag_wait": wait_share,
        "tiny_launch_us": floor_us,
        "graph_replay": graph_replay,
        "decode_variants": variants,
    }
    out["config"]["latency_us_quantiles"] = quant
    if not args.no_cpu:
        from oracle import ag_gemm as oag
        t0 = time.perf_counter()
        oag.ag_gemm(a, b, dtype="e4m3", a_scales=sa, b_scales=sb)
        dt = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": dt * 1e6, "unit": "us",
                               "cores": int(os.environ.get("OMP_NUM_THREADS", os.cpu_count())), "kind": "oracle",
                               "seconds": dt, "sample": "the whole workload (table decode + fp64 GEMM)"}
    return out


def bench_yardstick(args):
    """The tile engine against the vendor library's plain GEMM (hipBLASLt through torch.matmul) on the cfg 2 and
    cfg 3 shapes, N(0,1) / N(0,1/K) bf16 made on the device, B rotating through three copies.  The engine runs as
    ditron_ag_gemm with every shard resident and the flags preset (no communication on either side).  One
    step = the four launches once; `value` is the engine's geometric-mean TFLOP/s."""
    import math
    import torch
    from paper_2605_02953_amd import binding as B
    from gpu_util import AgGemmRun

    world, m_r = 8, 1024
    m = world * m_r
    problems = []
    for name, n, k in (("cfg2 shape", 3584, 8192), ("cfg3 shape", 8192, 3584)):
        a = torch.randn((m, k), device="cuda").to(torch.bfloat16)
        bs = [(torch.randn((n, k), device="cuda") * k ** -0.5).to(torch.bfloat16) for _ in range(3)]
        run = AgGemmRun(B, world, m_r, n, k)
        run.workspace.copy_(a.view(run.workspace.dtype))
        cnt = [0]

        def ours(run=run, bs=bs, cnt=cnt):
            cnt[0] += 1
            assert run(None, bs[cnt[0] % 3].view(torch.int16), 0, flags=B.FLAGS_PRESET) == B.OK

        def vendor(a=a, bs=bs, cnt=cnt):
            cnt[0] += 1
            torch.matmul(a, bs[cnt[0] % 3].t())

        problems.append((name, n, k, ours, vendor))

    def step():
        for pr in problems:
            pr[3]()
            pr[4]()

    _ramp(torch, step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    reps = max(1, args.steps)
    per = {}
    t0 = time.perf_counter()
    for _ in range(reps):
        for name, n, k, ours, vendor in problems:
            for who, fn in (("engine", ours), ("vendor", vendor)):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                fn()
                e1.record()
                per.setdefault((name, who), []).append((e0, e1))
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    rows, logs, flops_total = [], [], 0.0
    for name, n, k, _, _ in problems:
        flops = 2.0 * m * n * k
        row = {"shape": name, "m": m, "n": n, "k": k}
        for who in ("engine", "vendor"):
            us = _quantiles_us(per[(name, who)])["median"]
            row[who + "_us"] = us
            row[who + "_tflops"] = flops / us / 1e6
        flops_total += flops
        logs.append(math.log(row["engine_tflops"]))
        rows.append(row)
    value = math.exp(sum(logs) / len(logs))
    return {
        "metric": "TFLOP/s of the tile engine, flags preset (geometric mean over the cfg 2 and cfg 3 shapes), beside the vendor GEMM",
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": reps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / reps, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "yardstick: [8192, 3584, 8192] and [8192, 8192, 3584] bf16 GEMMs, B stored [n,k], engine vs torch.matmul"},
        "roofline": {"bound": "mfma", "achieved": value, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": value / PEAK_BF16_TFLOPS, "traffic": None, "kernel": "ag_gemm_kernel, flags preset"},
        "shapes": rows,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--no-cpu", action="store_true", help="skip the cpu_baseline leg")
    ap.add_argument("--weight-copies", type=int, default=3,
                    help="cfg2, cfg3, cfg5, gemm_ar: device copies of the weight operand B that the steps rotate through (1 = the same buffer every step)")
    ap.add_argument("--decode-variant", type=int, default=0, help="cfg5: kernel variant of the decode path (0 = library's choice)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU's share on one GPU; --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    calib, copy_gbs = _calibration_copy(torch)
    if args.workload in ("cfg1", "cfg2"):
        out = bench_ag_gemm(args, int(args.workload[3:]))
    elif args.workload == "cfg3":
        out = bench_gemm_rs(args)
    elif args.workload == "cfg4":
        out = bench_moe(args)
    elif args.workload == "cfg5":
        out = bench_fp8(args)
    elif args.workload == "gemm_ar":
        out = bench_gemm_ar(args)
    elif args.workload == "sweep":
        out = bench_sweep(args)
    elif args.workload == "moe_sweep":
        out = bench_moe_sweep(args)
    elif args.workload == "moe_rs":
        out = bench_moe_rs(args)
    elif args.workload == "yardstick":
        out = bench_yardstick(args)
    else:
        print(f"bench.py: unknown workload {args.workload}", file=sys.stderr)
        sys.exit(2)
    if LAST_QUANTILES is not None:
        out["config"].setdefault("latency_us_quantiles", LAST_QUANTILES)
    out["calibration_copy_bytes"] = calib
    out["plain_copy_gbs"] = copy_gbs   # read + write bytes of a 256 MiB torch copy / its best time: the HBM rate a simple kernel reaches
    out["clock_ramp_s"] = RAMP_SECONDS   # untimed load before the W warm-up steps
    print(json.dumps(out))


if __name__ == "__main__":
    main()
