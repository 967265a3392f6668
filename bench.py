#!/usr/bin/env python3
"""Benchmark of the md_hom hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-instances]

A step is one pass of the hot path (one library call: de-composition, scalar phase,
re-composition, including the second-pass combine where a reduction dimension is split)
over one batch of seeded synthetic input that is already resident in HBM.  The headline
line is the Jacobi-3D 512^3 configuration; the other configurations are measured the same
way and reported under "instances" in the same JSON line.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "per-instance GFLOP/s or GB/s and % of roofline on 1 MI355X"

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_FP32_MFMA_TFLOPS = 157.3
# Vector ALU: 256 CUs x 4 SIMDs x 32 lanes x 2.4 GHz = 78.6 T lane-op/s.  This is the width behind the
# published FP32 vector peak (157.3 TFLOP/s = 78.6 T fused multiply-adds a second), and no instruction
# kind issues faster: moves, 32-bit add / subtract, bitwise logic and fp32 add / multiply / FMA on
# vector-register operands measure 2.2-2.4 cycles per wavefront instruction, the other kinds (compare,
# select, min / max, three-operand and 24-bit multiply-add forms, anything with a scalar-register or
# inline-constant operand) 4.0-4.2 cycles, i.e. 16 lanes a cycle = 39.3 T lane-op/s.  A kernel bound
# by VALU issue is priced against the full width; the 16-lane figure and the measured rate of a
# register-resident loop of the kernel's own instruction mix are reported beside it.
PEAK_VALU_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12
PEAK_VALU_16LANE_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12

# Counter readings that bench.py quotes come from ONE tracked file, written by
# paper_2405_05118_amd/profile_summary.py from the same rocprofv3 --pmc runs as profiles/*.md:
#   traffic_bytes[workload]        HBM bytes per step (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy)
#   valu_insts_per_pair[workload]  SQ_INSTS_VALU x 64 / pairs of the custom-reduce kernels
with open(os.path.join(ROOT, "paper_2405_05118_amd", "measured_counters.json")) as _fh:
    MEASURED = json.load(_fh)
TRAFFIC_BYTES = MEASURED["traffic_bytes"]
VALU_PER_PAIR = MEASURED["valu_insts_per_pair"]

# Inputs of a step stay in the 256 MB last-level cache from one step to the next when the working set is
# smaller than that: such rows say so ("cache_resident"), and an HBM-bound row among them rotates through
# enough copies of its streamed operand that every step really reads it from HBM.
LLC_BYTES = 256 * 1024 * 1024


LAST_SPREAD = {}
MIN_WARM_MS = 0.0
ORACLE_SECONDS = 3.0  # host time the oracle gets per BASELINE row (a bounded sample of the workload)


# Student t, two-sided 99 %, by degrees of freedom (the next lower listed value is used)
_T99 = {9: 3.250, 14: 2.977, 19: 2.861, 24: 2.797, 29: 2.756, 39: 2.708, 49: 2.680, 59: 2.660, 79: 2.640, 99: 2.626}
ADAPTIVE = False       # per-instance table: keep timing until the 99 % confidence interval is within 5 %
CI_TARGET = 0.05
MAX_GROUPS = 100
MAX_TIMED_S = 4.0
GROUP_MS = 2.0


def _t99(dof):
    return _T99[max(k for k in _T99 if k <= dof)] if dof >= 9 else 3.250


def _events_ms(torch, fn, steps, warmup):
    """(events ms, wall ms) per step: `steps` launches bracketed by synchronize on both sides;
    HIP events on the launch stream give the device time, the host clock the whole-job time.
    Events recorded every steps/10 launches inside the same timed region give the spread of the
    per-step time (half-width of the 99 % confidence interval of the mean, relative), kept in
    LAST_SPREAD for the caller.  With ADAPTIVE set (the per-instance table, not the headline, which
    times exactly `steps`), further groups of steps/10 launches are timed until that half-width is
    within 5 % of the mean (the paper's protocol, Section "Experimental Setup"), up to MAX_GROUPS
    groups or MAX_TIMED_S seconds; every group counts in the reported time."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    # per-instance table only (the headline does exactly `warmup` steps): short kernels keep warming
    # up until MIN_WARM_MS of launches have run, so that a 10-60 us kernel is not timed while the
    # clocks still ramp after the host-side input generation
    t_w = time.perf_counter()
    while (time.perf_counter() - t_w) * 1e3 < MIN_WARM_MS:
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
    groups = 10 if steps >= 20 else 1
    per = steps // groups
    if ADAPTIVE:
        # group length from a pilot of five launches: about GROUP_MS of device time per group, so that a
        # group of 10 us kernels is not two launches long
        p0, p1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        p0.record()
        for _ in range(5):
            fn()
        p1.record()
        torch.cuda.synchronize()
        groups = 10
        per = int(max(2, min(200, GROUP_MS / max(p0.elapsed_time(p1) / 5, 1e-4))))
        steps = groups * per
    seg = []  # (start event, end event, launches) of every timed group

    def batch(sizes):
        """Time len(sizes) groups back to back; returns the host seconds around them."""
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(sizes) + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for g, n in enumerate(sizes):
            for _ in range(n):
                fn()
            ev[g + 1].record()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        seg.extend((ev[g], ev[g + 1], n) for g, n in enumerate(sizes))
        return dt

    wall_s = batch([per] * (groups - 1) + [steps - per * (groups - 1)])

    def spread():
        t = [a.elapsed_time(b) / n for a, b, n in seg]
        mean = sum(t) / len(t)
        var = sum((x - mean) ** 2 for x in t) / (len(t) - 1)
        return {"groups": len(t), "ci99_rel": _t99(len(t) - 1) * (var / len(t)) ** 0.5 / mean,
                "min_ms": min(t), "max_ms": max(t)}

    LAST_SPREAD.clear()
    if groups > 1:
        sp = spread()
        while ADAPTIVE and sp["ci99_rel"] > CI_TARGET and len(seg) < MAX_GROUPS and wall_s < MAX_TIMED_S:
            wall_s += batch([per] * 10)  # ten more groups, timed like the first ten; all of them count
            sp = spread()
        sp["steps_timed"] = sum(n for _, _, n in seg)
        sp["ci99_within_5pct"] = bool(sp["ci99_rel"] <= CI_TARGET)
        LAST_SPREAD.update(sp)
    total = sum(n for _, _, n in seg)
    dev_ms = sum(a.elapsed_time(b) for a, b, _ in seg)
    return dev_ms / total, wall_s * 1e3 / total


def _ws(torch, mdh, inst, sizes):
    n = mdh.mdh_workspace_size(inst, sizes)
    return torch.empty(max(n, 4) // 4, dtype=torch.int32, device="cuda") if n else None


def bench_stencil(torch, mdh, W, name, steps, warmup, cpu):
    cfg = W.CONFIGS[name]
    x = W.device_uniform(cfg.seed, 1, (cfg.nx + 2, cfg.ny + 2, cfg.nz + 2), 0.0, 1.0)
    out = torch.empty((cfg.nx, cfg.ny, cfg.nz), dtype=torch.float32, device="cuda")
    ms, wall = _events_ms(torch, lambda: mdh.mdh_stencil(x, out, cfg.c0, cfg.c1), steps, warmup)
    nbytes = 4 * ((cfg.nx + 2) * (cfg.ny + 2) * (cfg.nz + 2) + cfg.nx * cfg.ny * cfg.nz)
    gbs = nbytes / ms / 1e6
    res = {
        "value": nbytes / wall / 1e6, "unit": "GB/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "stencil_kernel",
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_bytes": nbytes,
    }
    if cpu:
        import numpy as np

        import oracle

        xh = x.cpu().numpy()
        oracle.jacobi3d(xh, cfg.c0, cfg.c1)  # untimed: first touch of the output pages
        sweeps, t0 = 0, time.perf_counter()
        while sweeps < 3 or time.perf_counter() - t0 < ORACLE_SECONDS:
            oracle.jacobi3d(xh, cfg.c0, cfg.c1)
            sweeps += 1
        dt = (time.perf_counter() - t0) / sweeps
        res["cpu_baseline"] = {"value": nbytes / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "whole %dx%dx%d grid, mean of %d sweeps (%.3f s each)" % (cfg.nx, cfg.ny, cfg.nz, sweeps, dt)}
        del xh, np
    return res


def _split_variant(mdh, sizes, S):
    """The default tile configuration with the reduction dimension split S ways over workgroups."""
    d = mdh.mdh_default_params(mdh.MDH_MATMUL, sizes)
    for i in range(mdh.mdh_num_candidates(mdh.MDH_MATMUL, sizes)):
        p = mdh.mdh_candidate(mdh.MDH_MATMUL, sizes, i)
        same_tile = all(list(p.prt[l][:3]) == list(d.prt[l][:3]) for l in (1, 2, 4, 5))
        if same_tile and p.prt[3][2] == S:
            return p
    return None


def bench_matmul(torch, mdh, W, name, steps, warmup, cpu, split=None):
    cfg = W.CONFIGS[name]
    sizes = (cfg.M, cfg.N, cfg.K)
    a = W.device_uniform(cfg.seed, 1, (cfg.M, cfg.K), -1.0, 1.0)
    b = W.device_uniform(cfg.seed, 2, (cfg.K, cfg.N), -1.0, 1.0)
    c = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device="cuda")
    p = mdh.mdh_default_params(mdh.MDH_MATMUL, sizes) if split is None else _split_variant(mdh, sizes, split)
    nws = mdh.mdh_workspace_size(mdh.MDH_MATMUL, sizes, p)
    ws = torch.empty(max(nws, 4) // 4, dtype=torch.int32, device="cuda") if nws else None
    ms, wall = _events_ms(torch, lambda: mdh.mdh_matmul(a, b, c, p, ws), steps, warmup)
    flop = 2.0 * cfg.M * cfg.N * cfg.K
    tf = flop / ms / 1e9
    res = {
        "value": flop / wall / 1e6, "unit": "GFLOP/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": ("matmul_ksplit16_kernel" if p.blk[0] == 16 else "matmul_ksplit_kernel" if p.prt[4][2] > 1 else "matmul_kernel")
        + (" + combine_sum_kernel" if p.prt[3][2] > 1 else ""),
        "wavefront_parts_of_k": int(p.prt[4][2]),
        "split_k": int(p.prt[3][2]),
        "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": TRAFFIC_BYTES.get(name if split is None else "%s_split_k%d" % (name, split))},
        "algorithmic_flop": flop,
        "algorithmic_bytes": 4 * (cfg.M * cfg.K + cfg.K * cfg.N + cfg.M * cfg.N),
        "cache_resident": 4 * (cfg.M * cfg.K + cfg.K * cfg.N + cfg.M * cfg.N) < LLC_BYTES,
    }
    if flop < 1e9:
        # launch-bound: the eager figure above is the rate at which this host issues launches; replayed from a
        # graph of 100 calls the same kernel runs back to back
        gms = _graph_ms_per_call(torch, lambda: mdh.mdh_matmul(a, b, c, p, ws))
        res["in_graph"] = {"ms_per_step": gms, "GFLOPs": flop / gms / 1e6, "frac": flop / gms / 1e9 / PEAK_FP32_MFMA_TFLOPS,
                           "calls_per_graph": 100}
    if cpu:
        import oracle

        # a probe of a few rows sizes the sample to about ORACLE_SECONDS of work (whole matrix if less)
        bh = b.cpu().numpy()
        rows = max(1, min(cfg.M, int(6e8 // (cfg.N * cfg.K))))
        t0 = time.perf_counter()
        oracle.matmul(a[:rows].cpu().numpy(), bh)
        probe = time.perf_counter() - t0
        rows = max(rows, min(cfg.M, int(rows * ORACLE_SECONDS / max(probe, 1e-6))))
        ah = a[:rows].cpu().numpy()
        reps, t0 = 0, time.perf_counter()
        while reps < 1 or (rows == cfg.M and time.perf_counter() - t0 < ORACLE_SECONDS):
            oracle.matmul(ah, bh)
            reps += 1
        dt = (time.perf_counter() - t0) / reps
        res["cpu_baseline"] = {"value": 2.0 * rows * cfg.N * cfg.K / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "first %d rows of C, %d time(s) (%.2f s each)" % (rows, reps, dt)}
    return res


def bench_mcc(torch, mdh, W, name, steps, warmup, cpu):
    cfg = W.CONFIGS[name]
    P = (cfg.H - cfg.R) // cfg.stride[0] + 1
    Q = (cfg.W - cfg.S) // cfg.stride[1] + 1
    x = W.device_normal(cfg.seed, 1, (cfg.N, cfg.H, cfg.W, cfg.C))
    f = W.device_normal(cfg.seed, 2, (cfg.K, cfg.R, cfg.S, cfg.C))
    o = torch.empty((cfg.N, P, Q, cfg.K), dtype=torch.float32, device="cuda")
    ws = _ws(torch, mdh, mdh.MDH_MCC, (cfg.N, P, Q, cfg.K, cfg.C, cfg.R, cfg.S, cfg.stride[0], cfg.stride[1]))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_mcc(x, f, o, cfg.stride, None, ws), steps, warmup)
    flop = 2.0 * cfg.N * P * Q * cfg.K * cfg.C * cfg.R * cfg.S
    tf = flop / ms / 1e9
    res = {
        "value": flop / wall / 1e6, "unit": "GFLOP/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "mcc_flat_kernel" if cfg.C <= 8 else "mcc_kernel",
        "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_FP32_MFMA_TFLOPS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_flop": flop,
        "algorithmic_bytes": 4 * (x.numel() + f.numel() + o.numel()),
        "cache_resident": 4 * (x.numel() + f.numel() + o.numel()) < LLC_BYTES,
    }
    if cpu:
        import numpy as np

        import oracle

        if cfg.C <= 8:
            xh, fh = x[:4].cpu().numpy(), f.cpu().numpy()  # four whole images
        else:
            xh, fh = x[:1].cpu().numpy(), f.cpu().numpy()  # image 0, every output row (a few seconds)
        dt, oreps, r = _oracle_seconds(lambda: oracle.mcc(np.ascontiguousarray(xh), fh, cfg.stride))
        res["cpu_baseline"] = {"value": 2.0 * r.size * cfg.C * cfg.R * cfg.S / dt / 1e9, "unit": "GFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "output rows p<%d of the first %d image(s), mean of %d call(s) (%.3f s each)" % (r.shape[1], r.shape[0], oreps, dt)}
    return res


def bench_prl(torch, mdh, W, name, steps, warmup, cpu):
    cfg = W.CONFIGS[name]
    sizes = (cfg.nA, cfg.nB, cfg.nF)
    alph = W.prl_alphabets(cfg.nF)
    A = torch.stack([W.device_integers(cfg.seed, 1 + 2 * f, (cfg.nA,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    B = torch.stack([W.device_integers(cfg.seed, 2 + 2 * f, (cfg.nB,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    wp = W.device_integers(cfg.seed, 40, (cfg.nF,), 1, W.PRL_WEIGHT_MAX)
    wm = W.device_integers(cfg.seed, 41, (cfg.nF,), -W.PRL_WEIGHT_MAX, 0)
    s = torch.empty(cfg.nA, dtype=torch.int32, device="cuda")
    i = torch.empty(cfg.nA, dtype=torch.int32, device="cuda")
    ws = _ws(torch, mdh, mdh.MDH_CUSTOM_REDUCE, sizes)
    before = valu_calibration(torch, mdh, kinds=("prl_fast_mix",))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_custom_reduce(A, B, wp, wm, s, i, None, ws), steps, warmup)
    after = valu_calibration(torch, mdh, kinds=("prl_fast_mix",))
    pairs = float(cfg.nA) * cfg.nB
    per_pair = VALU_PER_PAIR[name]  # SQ_INSTS_VALU of this kernel x 64 lanes / pairs
    tops = pairs * per_pair / ms / 1e9
    nbytes = 4 * (A.numel() + B.numel() + 2 * cfg.nF + 2 * cfg.nA)
    res = {
        "value": pairs / wall / 1e6, "unit": "Gpairs/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "i32",
        "kernel": "prl_fast_kernel + combine_maxidx_kernel",
        "roofline": _alu_roofline(tops, before, after, TRAFFIC_BYTES.get(name), "prl_fast_mix"),
        "lane_ops_per_pair": per_pair,
        "algorithmic_bytes": nbytes,
        "hbm_GBs_algorithmic": nbytes / ms / 1e6,
        "cache_resident": True,
    }
    if cpu:
        import oracle

        rows = list(range(0, cfg.nA, 4))  # every fourth record of A against all of B (a second or so)
        Ah, Bh = A.cpu().numpy(), B.cpu().numpy()
        t0 = time.perf_counter()
        oracle.custom_reduce_rows(Ah, Bh, wp.cpu().numpy(), wm.cpu().numpy(), rows)
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": len(rows) * cfg.nB / dt / 1e9, "unit": "Gpairs/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "%d records of A against all of B (%.2f s)" % (len(rows), dt)}
    return res


def bench_dot(torch, mdh, W, name, steps, warmup, cpu):
    K = 1 << 28
    seed = W.SEED_BASE + 7
    x = W.device_uniform(seed, 1, (K,), -1.0, 1.0)
    y = W.device_uniform(seed, 2, (K,), -1.0, 1.0)
    out = torch.empty(1, dtype=torch.float32, device="cuda")
    ws = _ws(torch, mdh, mdh.MDH_DOT, (K,))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_dot(x, y, out, None, ws), steps, warmup)
    nbytes = 8 * K
    gbs = nbytes / ms / 1e6
    res = {
        "value": nbytes / wall / 1e6, "unit": "GB/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "dot_kernel + dot_combine_kernel", "K": K,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_bytes": nbytes,
    }
    if cpu:
        import oracle

        n = 1 << 26
        xh, yh = x[:n].cpu().numpy(), y[:n].cpu().numpy()
        dt, oreps, _ = _oracle_seconds(lambda: oracle.dot(xh, yh))
        res["cpu_baseline"] = {"value": 8 * n / dt / 1e9, "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "first 2^26 elements, mean of %d call(s) (%.3f s each; the scalar reduction is sequential)" % (oreps, dt)}
    return res


def bench_matvec(torch, mdh, W, name, steps, warmup, cpu):
    M = K = 16384
    seed = W.SEED_BASE + 8
    A = W.device_uniform(seed, 1, (M, K), -1.0, 1.0)
    x = W.device_uniform(seed, 2, (K,), -1.0, 1.0)
    y = torch.empty(M, dtype=torch.float32, device="cuda")
    ws = _ws(torch, mdh, mdh.MDH_MATVEC, (M, K))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_matvec(A, x, y, None, ws), steps, warmup)
    nbytes = 4 * (M * K + K + M)
    gbs = nbytes / ms / 1e6
    res = {
        "value": nbytes / wall / 1e6, "unit": "GB/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "matvec_kernel", "M": M, "K": K,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_bytes": nbytes,
    }
    if cpu:
        import oracle

        rows = 4096
        Ah, xh = A[:rows].cpu().numpy(), x.cpu().numpy()
        dt, oreps, _ = _oracle_seconds(lambda: oracle.matvec(Ah, xh))
        res["cpu_baseline"] = {"value": 4 * rows * K / dt / 1e9, "unit": "GB/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "first %d rows, mean of %d call(s) (%.4f s each)" % (rows, oreps, dt)}
    return res


def bench_matmul_ex(torch, mdh, W, name, steps, warmup, cpu):
    """Small-M MatMul through the batched / transposed entry point (batch 1, no transposes)."""
    cfg = W.CONFIGS[name]
    sizes = (1, cfg.M, cfg.N, cfg.K, 0, 0, 0)
    a = W.device_uniform(cfg.seed, 1, (1, cfg.M, cfg.K), -1.0, 1.0)
    b = W.device_uniform(cfg.seed, 2, (1, cfg.K, cfg.N), -1.0, 1.0)
    c = torch.empty((1, cfg.M, cfg.N), dtype=torch.float32, device="cuda")
    p = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
    ws = _ws(torch, mdh, mdh.MDH_BMATMUL, sizes)
    flop = 2.0 * cfg.M * cfg.N * cfg.K
    nbytes = 4 * (cfg.M * cfg.K + cfg.K * cfg.N + cfg.M * cfg.N)
    # B is the operand that streams; when it would stay in the last-level cache from step to step, the
    # steps rotate through enough identical copies of it (twice the cache in total) to read it from HBM
    copies = 1 if 4 * b.numel() >= LLC_BYTES else -(-2 * LLC_BYTES // (4 * b.numel()))
    bs = [b] + [b.clone() for _ in range(copies - 1)]
    turn = [0]

    def step():
        turn[0] = (turn[0] + 1) % copies
        mdh.mdh_matmul_ex(a, bs[turn[0]], c, False, False, False, None, ws)

    ms, wall = _events_ms(torch, step, steps, warmup)
    gbs = nbytes / ms / 1e6
    # 2M/4 FLOP per byte of B: far below the ridge (19.7 FLOP/B), so B streaming from HBM is the bound
    res = {
        "value": flop / wall / 1e6, "unit": "GFLOP/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "matmul_ex / skinny kernel + combine", "split_k": int(p.prt[3][3]),
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_flop": flop,
        "algorithmic_bytes": nbytes,
        "rotating_copies_of_B": copies,
    }
    if cpu:
        import oracle

        cols = max(1, min(cfg.N, int(4e8 // (cfg.M * cfg.K))))
        ah, bh = a[0].cpu().numpy(), b[0, :, :cols].contiguous().cpu().numpy()
        dt, oreps, _ = _oracle_seconds(lambda: oracle.matmul(ah, bh))
        res["cpu_baseline"] = {"value": 2.0 * cfg.M * cols * cfg.K / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "first %d columns of C, mean of %d call(s) (%.4f s each)" % (cols, oreps, dt)}
    return res


def bench_bmatmul(torch, mdh, W, name, steps, warmup, cpu):
    """bMatMul / MatMul^T on the LDS-tiled MFMA kernel of the batched / transposed entry point."""
    cfg = W.CONFIGS[name]
    ta, tb, tc = cfg.trans
    sizes = (cfg.batch, cfg.M, cfg.N, cfg.K, ta, tb, tc)
    a = W.device_uniform(cfg.seed, 1, (cfg.batch, cfg.K, cfg.M) if ta else (cfg.batch, cfg.M, cfg.K), -1.0, 1.0)
    b = W.device_uniform(cfg.seed, 2, (cfg.batch, cfg.N, cfg.K) if tb else (cfg.batch, cfg.K, cfg.N), -1.0, 1.0)
    c = torch.empty((cfg.batch, cfg.N, cfg.M) if tc else (cfg.batch, cfg.M, cfg.N), dtype=torch.float32, device="cuda")
    p = mdh.mdh_default_params(mdh.MDH_BMATMUL, sizes)
    ws = _ws(torch, mdh, mdh.MDH_BMATMUL, sizes)
    ms, wall = _events_ms(torch, lambda: mdh.mdh_matmul_ex(a, b, c, bool(ta), bool(tb), bool(tc), None, ws), steps, warmup)
    flop = 2.0 * cfg.batch * cfg.M * cfg.N * cfg.K
    tf = flop / ms / 1e9
    res = {
        "value": flop / wall / 1e6, "unit": "GFLOP/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "matmul_ex_kernel", "split_k": int(p.prt[3][3]),
        "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_FP32_MFMA_TFLOPS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_flop": flop,
        "algorithmic_bytes": 4 * cfg.batch * (cfg.M * cfg.K + cfg.K * cfg.N + cfg.M * cfg.N),
    }
    if cpu:
        import oracle

        # batch 0, the first rows of C: the views are undone on the host, the oracle sees plain A and B
        rows = max(1, min(cfg.M, int(4e8 // (cfg.N * cfg.K))))
        a0 = a[0].t() if ta else a[0]
        b0 = b[0].t() if tb else b[0]
        ah, bh = a0[:rows].contiguous().cpu().numpy(), b0.contiguous().cpu().numpy()
        dt, oreps, _ = _oracle_seconds(lambda: oracle.matmul(ah, bh))
        res["cpu_baseline"] = {"value": 2.0 * rows * cfg.N * cfg.K / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.num_threads(),
                               "kind": "oracle", "sample": "batch 0, first %d rows of C, mean of %d call(s) (%.3f s each)" % (rows, oreps, dt)}
    return res


def bench_capsule(torch, mdh, W, name, steps, warmup, cpu):
    """MCC_Capsule at the first-layer shape of ResNet-50 (training): MCC on 4 x 4 matrices."""
    cfg = W.CONFIGS["mcc_resnet50_first"]
    P = (cfg.H - cfg.R) // cfg.stride[0] + 1
    Q = (cfg.W - cfg.S) // cfg.stride[1] + 1
    x = W.device_normal(cfg.seed + 100, 1, (cfg.N, cfg.H, cfg.W, cfg.C, 4, 4))
    f = W.device_normal(cfg.seed + 100, 2, (cfg.K, cfg.R, cfg.S, cfg.C, 4, 4))
    o = torch.empty((cfg.N, P, Q, cfg.K, 4, 4), dtype=torch.float32, device="cuda")
    ms, wall = _events_ms(torch, lambda: mdh.mdh_mcc_capsule(x, f, o, cfg.stride), steps, warmup)
    flop = 2.0 * cfg.N * P * Q * cfg.K * cfg.C * cfg.R * cfg.S * 64
    tf = flop / ms / 1e9
    res = {
        "value": flop / wall / 1e6, "unit": "GFLOP/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": "capsule_kernel",
        "roofline": {"bound": "mfma", "achieved": tf, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": tf / PEAK_FP32_MFMA_TFLOPS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_flop": flop,
        "algorithmic_bytes": 4 * (x.numel() + f.numel() + o.numel()),
    }
    if cpu:
        import numpy as np

        import oracle

        xh, fh = x[:1, : cfg.R + 2 * 7].cpu().numpy(), f.cpu().numpy()  # 8 output rows of image 0
        dt, oreps, r = _oracle_seconds(lambda: oracle.mcc_capsule(np.ascontiguousarray(xh), fh, cfg.stride))
        res["cpu_baseline"] = {"value": 2.0 * r.size * cfg.C * cfg.R * cfg.S * 4 / dt / 1e9, "unit": "GFLOP/s",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "output rows p<%d of image 0, mean of %d call(s) (%.3f s each)" % (r.shape[1], oreps, dt)}
    return res


def bench_scan(torch, mdh, W, name, steps, warmup, cpu):
    """Row-wise scan(+): one long row (chunks over workgroups) or many rows (a workgroup per row)."""
    R, n = (1, 1 << 28) if name == "scan_2p28" else (65536, 4096)
    seed = W.SEED_BASE + 12
    x = W.device_uniform(seed, 1, (R, n), -1.0, 1.0)
    out = torch.empty_like(x)
    ws = _ws(torch, mdh, mdh.MDH_SCAN, (R, n))
    p = mdh.mdh_default_params(mdh.MDH_SCAN, (R, n))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_scan(x, out, None, ws), steps, warmup)
    assert not mdh.mdh_scan_timed_out(x, None, ws), "a bounded wait of the single-pass scan expired: results invalid"
    nbytes = 8 * R * n  # every element read once and written once
    gbs = nbytes / ms / 1e6
    chunks = int(p.prt[3][1])
    single_pass = chunks > 1 and int(p.in_region[0]) == 2  # the chunk waits in registers (MDH_MR_VGPR)
    res = {
        "value": nbytes / wall / 1e6, "unit": "GB/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "f32",
        "kernel": ("scan_row_resident_kernel (the row stays in registers)" if chunks == 1 and int(p.prt[2][1]) > 4 else
                   "scan_apply_kernel" if chunks == 1 else
                   "scan_onepass_init_kernel + scan_onepass_kernel (single pass)" if single_pass else
                   "scan_totals_kernel + scan_offsets_kernel + scan_apply_kernel"),
        "rows": R, "n": n, "chunks_per_row": chunks,
        "roofline": {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                     "frac": gbs / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES.get(name)},
        "algorithmic_bytes": nbytes,
        "kernel_bytes": nbytes + (4 * R * n if chunks > 1 and not single_pass else 0),  # three kernels read the input twice
    }
    if cpu:
        import oracle

        rows = max(1, min(R, (1 << 26) // n))
        cols = min(n, 1 << 26)
        xh = x[:rows, :cols].contiguous().cpu().numpy()
        dt, oreps, _ = _oracle_seconds(lambda: oracle.scan_rows(xh))
        res["cpu_baseline"] = {"value": 8 * rows * cols / dt / 1e9, "unit": "GB/s", "cores": min(rows, oracle.num_threads()),
                               "kind": "oracle", "sample": "first %d row(s) x %d columns, mean of %d call(s) (%.3f s each)" % (rows, cols, oreps, dt)}
    return res


def bench_histo_generic(torch, mdh, W, name, steps, warmup, cpu):
    """Histo through the generic runtime-compiled path: md_hom(f_Histo, (++, +)) over (bins, elements)."""
    nb, ne = 256, 1 << 24
    seed = W.SEED_BASE + 13
    elems = W.device_integers(seed, 1, (ne,), 0, nb - 1)
    bins = torch.arange(nb, dtype=torch.int32, device="cuda")
    out = torch.empty(nb, dtype=torch.int32, device="cuda")
    desc = mdh.custom_desc((nb, ne), (0, 1), ["int", "int"], [(0, "i1"), (1, "i0")], "int", 4,
                           "r = a0 == a1 ? 1 : 0;", "r = x + y;")
    op = mdh.mdh_custom_create(desc)
    n = mdh.mdh_custom_workspace_size(op)
    ws = torch.empty(max(n, 4), dtype=torch.uint8, device="cuda") if n else None
    before = valu_calibration(torch, mdh, kinds=("cmp_select",))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_custom_run(op, [elems, bins], out, ws), steps, warmup)
    after = valu_calibration(torch, mdh, kinds=("cmp_select",))
    pairs = float(nb) * ne
    # per (bin, element) pair at least a compare and a conditional add: 2 lane-ops
    tops = pairs * 2.0 / ms / 1e9
    res = {
        "value": pairs / wall / 1e6, "unit": "Gpairs/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "i32",
        "kernel": "mdh_custom_main + mdh_custom_combine (hipRTC)", "bins": nb, "elements": ne,
        "roofline": _alu_roofline(tops, before, after, TRAFFIC_BYTES.get(name), "cmp_select"),
        "lane_ops_per_pair": 2.0,
        "algorithmic_bytes": 4 * (ne + 2 * nb),
        "cache_resident": True,
    }
    if cpu:
        import numpy as np

        from oracle import instances as G

        m = 4096
        eh = elems[:m].cpu().numpy().tolist()
        t0 = time.perf_counter()
        G.histo(eh, list(range(16)))
        dt = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": 16 * m / dt / 1e9, "unit": "Gpairs/s", "cores": 1, "kind": "oracle",
                               "sample": "generic evaluator, 16 bins x %d elements (%.2f s)" % (m, dt)}
        del np
    mdh.mdh_custom_destroy(op)
    return res


def bench_prl_generic(torch, mdh, W, name, steps, warmup, cpu):
    """The custom reduce again, this time through the generic path: record and result types, wght and
    max_idx given as source and compiled at run time (same inputs and sizes as prl_2p16_2p18)."""
    cfg = W.CONFIGS["prl_2p16_2p18"]
    alph = W.prl_alphabets(cfg.nF)
    A = torch.stack([W.device_integers(cfg.seed, 1 + 2 * f, (cfg.nA,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    B = torch.stack([W.device_integers(cfg.seed, 2 + 2 * f, (cfg.nB,), 0, a - 1) for f, a in enumerate(alph)], 1).contiguous()
    wp = W.device_integers(cfg.seed, 40, (cfg.nF,), 1, W.PRL_WEIGHT_MAX)
    wm = W.device_integers(cfg.seed, 41, (cfg.nF,), -W.PRL_WEIGHT_MAX, 0)
    out = torch.empty((cfg.nA, 2), dtype=torch.int32, device="cuda")
    pre = "struct rec { int f[8]; }; struct res { int score; int idx; };"
    fsrc = ("int s = 0; for (int k = 0; k < 8; ++k) s += a0.f[k] == a1.f[k] ? a2.f[k] : a3.f[k];"
            " r.score = s; r.idx = (int)i1;")
    osrc = "if (x.score > y.score || (x.score == y.score && x.idx < y.idx)) r = x; else r = y;"
    desc = mdh.custom_desc((cfg.nA, cfg.nB), (0, 1), ["rec"] * 4, [(0, "i0"), (1, "i1"), (2, "0"), (3, "0")], "res", 8,
                           fsrc, osrc, pre, fast_dim=0)
    op = mdh.mdh_custom_create(desc)
    n = mdh.mdh_custom_workspace_size(op)
    ws = torch.empty(max(n, 4), dtype=torch.uint8, device="cuda") if n else None
    before = valu_calibration(torch, mdh, kinds=("prl_mix",))
    ms, wall = _events_ms(torch, lambda: mdh.mdh_custom_run(op, [A, B, wp, wm], out, ws), steps, warmup)
    after = valu_calibration(torch, mdh, kinds=("prl_mix",))
    pairs = float(cfg.nA) * cfg.nB
    per_pair = VALU_PER_PAIR[name]  # this kernel's own SQ_INSTS_VALU x 64 lanes / pairs
    tops = pairs * per_pair / ms / 1e9
    res = {
        "value": pairs / wall / 1e6, "unit": "Gpairs/s", "ms_per_step": wall, "kernel_ms": ms, "dtype": "i32",
        "kernel": "mdh_custom_main + mdh_custom_combine (hipRTC)",
        "roofline": _alu_roofline(tops, before, after, TRAFFIC_BYTES.get(name)),
        "lane_ops_per_pair": per_pair,
        "cache_resident": True,
    }
    mdh.mdh_custom_destroy(op)
    return res


VALU_KINDS = {"xor_max": 0, "cmp_select": 1, "add3": 2, "prl_mix": 3, "fma_f32_vgpr": 4, "add_u32_vgpr": 5, "prl_fast_mix": 6}
_CAL_BUFS = {}


def valu_calibration(torch, mdh, kinds=tuple(VALU_KINDS)):
    """Issue rate (T lane-op/s) of the register-resident loop of each instruction kind, the shader clock
    read inside the kernel, and from both the issue cost in shader-clock cycles per wavefront
    instruction and SIMD.  Five launches each, HIP events on the launch stream."""
    B = mdh.binding
    if not _CAL_BUFS:
        g = torch.Generator(device="cpu").manual_seed(7)
        w = torch.cat([torch.randint(1, 1 << 16, (8,), generator=g), -torch.randint(0, 1 << 16, (8,), generator=g),
                       torch.randint(0, 16, (256 * 2 * 8,), generator=g)]).to(torch.int32)
        _CAL_BUFS.update(out=torch.empty(B.MDH_CALIB_BLOCKS * 256, dtype=torch.int32, device="cuda"),
                         w=w.cuda(), clk=torch.zeros(2, dtype=torch.int64, device="cuda"),
                         hz=mdh.mdh_calib_realtime_hz())
    out, w, clk, hz = _CAL_BUFS["out"], _CAL_BUFS["w"], _CAL_BUFS["clk"], _CAL_BUFS["hz"]
    res = {}
    for k in kinds:
        ops = [0]

        def run():
            ops[0] = mdh.mdh_calib_valu_kind(VALU_KINDS[k], out, 2048 if k == "prl_fast_mix" else 8192, w, clk)

        run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            run()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        c = clk.cpu().tolist()
        ghz = c[0] / c[1] * hz / 1e9 if c[1] > 0 and hz > 0 else None
        rate = ops[0] / ms / 1e9
        res[k] = {"Tlaneops": rate, "shader_clock_GHz": ghz,
                  # wavefront instructions per second and SIMD = rate / 64 lanes / 1024 SIMDs
                  "cycles_per_wave_inst": ghz * 1e9 / (rate * 1e12 / 64 / 1024) if ghz else None}
    return res


def _alu_roofline(tops, before, after, traffic, kind="prl_mix"):
    """Roofline object of a VALU-issue-bound row: the peak is the full vector-ALU width (32 lanes a cycle
    and SIMD at 2.4 GHz, the width of the published FP32 vector peak), which no instruction kind
    exceeds; beside it the 16-lane figure that the compare / select / min / max kinds are held to, and
    the measured rate of a register-resident loop of the same instruction kinds taken right before and
    right after the timed region, with the shader clock read inside that loop."""
    loop = max(before[kind]["Tlaneops"], after[kind]["Tlaneops"])
    return {"bound": "alu", "achieved": tops, "peak": PEAK_VALU_TOPS, "unit": "Tlane-op/s", "frac": tops / PEAK_VALU_TOPS,
            "traffic": traffic, "peak_16_lanes": PEAK_VALU_16LANE_TOPS, "frac_of_16_lanes": tops / PEAK_VALU_16LANE_TOPS,
            "same_kinds_loop_Tlaneops": loop, "same_kinds_loop": kind,
            "shader_clock_GHz": after[kind]["shader_clock_GHz"],
            "cycles_per_wave_inst": (after[kind]["shader_clock_GHz"] or 2.4) * 1e9 / (tops * 1e12 / 64 / 1024)}


def calibration(torch, mdh):
    """Attainable rates of this chip on the resources that bound the instances, from the library's
    calibration kernels (HIP events on the launch stream, 20 launches each)."""
    n = 256 * 1024 * 1024  # 1 GiB of fp32: four times the 256 MB last-level cache
    src = torch.ones(n, dtype=torch.float32, device="cuda")
    dst = torch.empty(n // 2, dtype=torch.float32, device="cuda")
    out = torch.empty(mdh.binding.MDH_CALIB_BLOCKS * 256, dtype=torch.float32, device="cuda")
    outi = torch.empty(mdh.binding.MDH_CALIB_BLOCKS * 256, dtype=torch.int32, device="cuda")
    res = {}
    ms, _ = _events_ms(torch, lambda: mdh.mdh_calib_copy(src[: n // 2], dst), 20, 3)
    res["copy_GBs"] = 2 * 4 * (n // 2) / ms / 1e6
    ms, _ = _events_ms(torch, lambda: mdh.mdh_calib_read(src, out), 20, 3)
    res["read_GBs"] = 4 * n / ms / 1e6
    flop = [0]

    def mf():
        flop[0] = mdh.mdh_calib_mfma(out, 4096)

    ms, _ = _events_ms(torch, mf, 20, 3)
    res["fp32_mfma_TFLOPs"] = flop[0] / ms / 1e9
    # 16 MFMAs x 64 cycles per iteration, 8 wavefronts per SIMD one after the other
    res["clock_GHz_under_mfma"] = 4096 * 16 * 64 * (mdh.binding.MDH_CALIB_BLOCKS * 4 / 1024) / ms / 1e6
    ops = [0]

    def va():
        ops[0] = mdh.mdh_calib_valu(outi, 16384)

    ms, _ = _events_ms(torch, va, 20, 3)
    res["int_valu_Tlaneops"] = ops[0] / ms / 1e9
    res["int_valu_by_kind"] = valu_calibration(torch, mdh)
    res["peaks"] = {"hbm_GBs": PEAK_HBM_GBS, "fp32_mfma_TFLOPs": PEAK_FP32_MFMA_TFLOPS,
                    "valu_Tlaneops": PEAK_VALU_TOPS, "valu_16_lanes_Tlaneops": PEAK_VALU_16LANE_TOPS}
    del src, dst, out, outi
    torch.cuda.empty_cache()
    return res


# the benchmark's five configurations (config 3 is two shapes) and the split-k line of the tall-skinny one
BASELINE_ROWS = ("matmul_256", "jacobi3d_512", "matmul_4096", "matmul_ts", "matmul_ts_split_k4", "mcc_resnet",
                 "prl_2p16_2p18")


def _graph_ms_per_call(torch, call, calls=100, reps=20):
    """Per-call time of `calls` launches captured once into a HIP graph and replayed (the entry points
    allocate nothing and synchronise nothing, so they can be captured after one eager call): what a
    launch-bound kernel costs when the host is out of the way."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        for _ in range(3):
            call()
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        for _ in range(calls):
            call()
    torch.cuda.synchronize()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (reps * calls)


def _oracle_seconds(fn, min_total=0.5, max_reps=200):
    """Mean time of one oracle call: repeated until min_total seconds have been spent (a sample of a few
    milliseconds would be timer noise), never tuned."""
    reps, t0 = 0, time.perf_counter()
    while True:
        out = fn()
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= min_total or reps >= max_reps:
            return dt / reps, reps, out


def _rounded(x):
    """Floats to 6 significant digits (keeps the one JSON line short); everything else unchanged."""
    if isinstance(x, float):
        return float("%.6g" % x)
    if isinstance(x, dict):
        return {k: _rounded(v) for k, v in x.items()}
    if isinstance(x, (list, tuple)):
        return [_rounded(v) for v in x]
    return x


def bench_matmul_ts_split(torch, mdh, W, name, steps, warmup, cpu):
    """The tall-skinny MatMul with the reduction dimension split four ways over workgroups (partial
    results in a device-memory workspace + second-pass combine)."""
    return bench_matmul(torch, mdh, W, "matmul_ts", steps, warmup, False, split=4)


BENCHES = {
    "dot_2p28": bench_dot,
    "matvec_16384": bench_matvec,
    "jacobi3d_512": bench_stencil,
    "matmul_4096": bench_matmul,
    "matmul_ts": bench_matmul,
    "matmul_ts_split_k4": bench_matmul_ts_split,
    "mcc_resnet": bench_mcc,
    "prl_2p16_2p18": bench_prl,
    "matmul_256": bench_matmul,
    "mcc_resnet50_first": bench_mcc,
    "matmul_resnet50_fc": bench_matmul_ex,
    "matmul_vgg16_fc": bench_matmul_ex,
    "bmatmul_16x1024": bench_bmatmul,
    "matmul_t_4096": bench_bmatmul,
    "mcc_capsule_resnet50_first": bench_capsule,
    "scan_2p28": bench_scan,
    "scan_rows_65536x4096": bench_scan,
    "histo_generic_256x2p24": bench_histo_generic,
    "prl_generic_2p16_2p18": bench_prl_generic,
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="jacobi3d_512", choices=sorted(BENCHES))
    ap.add_argument("--no-instances", action="store_true", help="measure only --workload")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="run a 512 MiB device copy first (reference kernel for --pmc byte counters)")
    ap.add_argument("--valu-kinds", action="store_true",
                    help="run the register-resident VALU loop of every instruction kind once first (for --pmc runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
                         "use --gpus 1\n")
        return 2

    import torch

    import paper_2405_05118_amd as mdh
    from paper_2405_05118_amd import workloads as W

    if not torch.cuda.is_available():
        sys.stderr.write("bench.py needs the GPU (and libmdh.so); there is no CPU fallback\n")
        return 3
    torch.cuda.set_device(0)
    mdh.lib()

    if args.calibration_copy:
        # a plain device copy of known size (512 MiB read + 512 MiB written), outside every timed
        # region: the reference the FETCH_SIZE / WRITE_SIZE counters of a --pmc run are scaled by
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
        torch.cuda.empty_cache()

    if args.valu_kinds:
        valu_calibration(torch, mdh)

    torch.cuda.synchronize()
    head = BENCHES[args.workload](torch, mdh, W, args.workload, args.steps, args.warmup, not args.no_cpu)
    head["spread"] = dict(LAST_SPREAD)
    torch.cuda.synchronize()
    torch.cuda.empty_cache()

    line = {
        "metric": METRIC,
        "value": head["value"],
        "unit": head["unit"],
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": head["dtype"],
        "data": "synthetic",
        "config": {"workload": args.workload, "params": "library default"},
        "roofline": head["roofline"],
    }
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    line["detail"] = {k: v for k, v in head.items() if k not in ("roofline", "cpu_baseline", "value", "unit")}

    if not args.no_instances:
        global MIN_WARM_MS, ADAPTIVE
        MIN_WARM_MS = 20.0
        ADAPTIVE = True  # keep timing each instance until the 99 % confidence interval is within 5 %
        inst = {}
        # the BASELINE configurations come last, so that they survive in a record that keeps only the
        # end of this line
        order = [n for n in BENCHES if n not in BASELINE_ROWS] + [n for n in BASELINE_ROWS if n in BENCHES]
        for name in order:
            if name == args.workload:
                continue
            inst[name] = BENCHES[name](torch, mdh, W, name, 20, max(2, min(args.warmup, 5)), not args.no_cpu)
            inst[name]["spread"] = dict(LAST_SPREAD)
            torch.cuda.synchronize()
            torch.cuda.empty_cache()
        ADAPTIVE = False
        line["calibration"] = calibration(torch, mdh)
        line["instances"] = inst
        # compact table of the BASELINE configurations (and the split-k line), last in the line:
        # [value, unit, ms_per_step, roofline.frac, roofline.bound, cpu_baseline value or null, ci99_rel]
        rows = {}
        everything = dict(inst)
        everything[args.workload] = head
        for name in BASELINE_ROWS:
            r = everything.get(name)
            if r is not None:
                rows[name] = [r["value"], r["unit"], r["ms_per_step"], r["roofline"]["frac"], r["roofline"]["bound"],
                              r.get("cpu_baseline", {}).get("value"), r.get("spread", {}).get("ci99_rel")]
                if "in_graph" in r:  # launch-bound row: ms per step and roofline fraction when replayed from a graph
                    rows[name] += [r["in_graph"]["ms_per_step"], r["in_graph"]["frac"]]
        line["baseline_rows"] = rows

    print(json.dumps(_rounded(line)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
