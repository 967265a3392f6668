#!/usr/bin/env python3
"""Turns rocprofv3 output of bench.py into the summaries under profiles/ and the counter file bench.py reads.

The profiling itself is four rocprofv3 passes per workload (the commands are written into every summary);
each pass runs `bench.py --workload W --no-instances --no-cpu`, so that every library kernel of a pass
belongs to workload W:

    D=<directory for the raw profiler output>
    for W in $(python3 -m paper_2405_05118_amd.profile_summary --workloads); do
      rocprofv3 --kernel-trace --stats --output-format csv -d $D/trace/$W -o p -- python3 bench.py --workload $W --no-instances --no-cpu --steps 50 --warmup 5
      rocprofv3 --pmc FETCH_SIZE --output-format csv -d $D/fetch/$W -o p -- python3 bench.py --workload $W --no-instances --no-cpu --steps 5 --warmup 1 --calibration-copy
      rocprofv3 --pmc WRITE_SIZE --output-format csv -d $D/write/$W -o p -- python3 bench.py --workload $W --no-instances --no-cpu --steps 5 --warmup 1 --calibration-copy
      rocprofv3 --pmc SQ_INSTS_VALU_MFMA_MOPS_F32 SQ_VALU_MFMA_BUSY_CYCLES SQ_BUSY_CYCLES SQ_WAVE_CYCLES SQ_INSTS_LDS SQ_LDS_BANK_CONFLICT SQ_INSTS_VALU SQ_WAIT_INST_ANY GRBM_GUI_ACTIVE --output-format csv -d $D/sq/$W -o p -- python3 bench.py --workload $W --no-instances --no-cpu --steps 5 --warmup 1 --valu-kinds
    done
    python3 -m paper_2405_05118_amd.profile_summary $D

The byte counters are scaled by what the same counter reads for the plain 512 MiB device copy that
`--calibration-copy` runs first (FETCH_SIZE counts in units that make that copy read half its size).
Output: three tables as text under profiles/ (kernel trace; HBM traffic; MFMA / LDS / VALU counters),
each with one line per (workload, kernel), and paper_2405_05118_amd/measured_counters.json (HBM bytes
per step; VALU instructions per pair of the custom-reduce kernels) -- the one place bench.py takes
counter readings from.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import statistics as st
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)

# algorithmic bytes per step (what the roofline of an HBM-bound row is priced with), by workload
ALG_BYTES = {
    "jacobi3d_512": 4 * (514 ** 3 + 512 ** 3),
    "dot_2p28": 8 << 28,
    "matvec_16384": 4 * (16384 * 16384 + 2 * 16384),
    "matmul_256": 4 * 3 * 256 * 256,
    "matmul_4096": 4 * 3 * 4096 * 4096,
    "matmul_ts": 4 * (65536 * 4096 + 4096 * 64 + 65536 * 64),
    "matmul_ts_split_k4": 4 * (65536 * 4096 + 4096 * 64 + 65536 * 64),
    "mcc_resnet": 4 * (16 * 230 * 230 * 64 + 128 * 49 * 64 + 16 * 224 * 224 * 128),
    "prl_2p16_2p18": 4 * ((1 << 16) * 8 + (1 << 18) * 8 + 16 + 2 * (1 << 16)),
    "prl_generic_2p16_2p18": 4 * ((1 << 16) * 8 + (1 << 18) * 8 + 16 + 2 * (1 << 16)),
    "mcc_resnet50_first": 4 * (16 * 230 * 230 * 3 + 64 * 49 * 3 + 16 * 112 * 112 * 64),
    "matmul_resnet50_fc": 4 * (16 * 2048 + 2048 * 1000 + 16 * 1000),
    "matmul_vgg16_fc": 4 * (16 * 25088 + 25088 * 4096 + 16 * 4096),
    "bmatmul_16x1024": 4 * 16 * 3 * 1024 * 1024,
    "matmul_t_4096": 4 * 3 * 4096 * 4096,
    "mcc_capsule_resnet50_first": 4 * 16 * (16 * 230 * 230 * 3 + 64 * 49 * 3 + 16 * 112 * 112 * 64),
    "scan_2p28": 8 << 28,
    "scan_rows_65536x4096": 8 << 28,
    "histo_generic_256x2p24": 4 * ((1 << 24) + 512),
}
PAIRS = {"prl_2p16_2p18": float(1 << 34), "prl_generic_2p16_2p18": float(1 << 34)}


def is_ours(name: str) -> bool:
    return "mdh::" in name or name.startswith("mdh_custom") or "mdh_custom" in name


def short(name: str) -> str:
    n = name.replace("void ", "").replace("mdh::(anonymous namespace)::", "")
    return n.split("(")[0]


def read_csv(pattern: str):
    files = glob.glob(pattern)
    return list(csv.DictReader(open(files[0]))) if files else []


def trace(root: str, wl: str):
    """(kernel, workgroups) -> list of durations in ns, skipping the warm-up launches of the pass."""
    rows = read_csv(os.path.join(root, "trace", wl, "*kernel_trace.csv"))
    rows.sort(key=lambda r: int(r["Start_Timestamp"]))
    g = collections.OrderedDict()
    for r in rows:
        if not is_ours(r["Kernel_Name"]):
            continue
        wgs = int(r["Grid_Size_X"]) * int(r.get("Grid_Size_Y", 1) or 1) // max(1, int(r["Workgroup_Size_X"]))
        g.setdefault((short(r["Kernel_Name"]), wgs), []).append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
    return g


def counters(root: str, what: str, wl: str):
    """(kernel, workgroups) -> {counter: mean per dispatch}; plus the reading of the reference copy."""
    rows = read_csv(os.path.join(root, what, wl, "*counter_collection.csv"))
    g = collections.OrderedDict()
    ref = collections.defaultdict(list)
    for r in rows:
        name = r["Kernel_Name"]
        if "rocclr_copyBuffer" in name:
            ref[r["Counter_Name"]].append(float(r["Counter_Value"]))
        if not is_ours(name):
            continue
        wgs = int(r["Grid_Size"]) // max(1, int(r["Workgroup_Size"]))
        g.setdefault((short(name), wgs), collections.defaultdict(list))[r["Counter_Name"]].append(float(r["Counter_Value"]))
    out = collections.OrderedDict((k, {c: st.mean(x) for c, x in v.items()}) for k, v in g.items())
    return out, {c: max(x) for c, x in ref.items()}


def main(argv):
    sys.path.insert(0, ROOT)
    if "--workloads" in argv:
        import bench

        print(" ".join(bench.BENCHES))
        return 0
    if len(argv) < 2:
        sys.stderr.write("usage: python3 -m paper_2405_05118_amd.profile_summary <directory of the raw profiler output> | --workloads\n")
        return 2
    root = argv[1]
    shown = os.path.relpath(os.path.abspath(root), ROOT)  # as the summaries print it in their commands
    workloads = sorted(os.path.basename(d) for d in glob.glob(os.path.join(root, "trace", "*")))
    if not workloads:
        sys.stderr.write("no passes under %s\n" % root)
        return 2
    cmd = "python3 bench.py --workload W --no-instances --no-cpu"
    # ---- kernel trace
    lines = []
    step_ns = {}
    for wl in workloads:
        total = 0.0
        for (k, wgs), v in trace(root, wl).items():
            v = v[len(v) // 10:]  # the first tenth of the launches are warm-up
            lines.append("| %s | %s | %d | %d | %d | %d | %d | %d |" % (wl, k, wgs, len(v), round(st.mean(v)), min(v), max(v), round(st.pstdev(v))))
            if "calib" not in k:
                total += st.mean(v)
        step_ns[wl] = total
    with open(os.path.join(ROOT, "profiles", "all_workloads_kernel_trace.md"), "w") as fh:
        fh.write("# rocprofv3 kernel trace: every kernel of every bench.py workload (MI355X, gfx950)\n\n"
                 "One pass per workload W (from the repository root on the GPU box):\n\n"
                 "    rocprofv3 --kernel-trace --stats --output-format csv -d " + shown + "/trace/W -o p -- " + cmd + " --steps 50 --warmup 5\n\n"
                 "Per-dispatch durations (ns) from the kernel trace, warm-up launches dropped; a workload with a split\n"
                 "reduction shows its second-pass kernel on a line of its own.  `bench.py` itself times the same launches\n"
                 "with HIP events on the launch stream (`kernel_ms` = all kernels of a step plus the gaps between them).\n\n"
                 "| workload | kernel | workgroups | dispatches | average ns | min ns | max ns | stddev |\n|---|---|---|---|---|---|---|---|\n"
                 + "\n".join(lines) + "\n")
    # ---- HBM traffic
    lines = []
    traffic = {}
    scale_note = ""
    for wl in workloads:
        f, fref = counters(root, "fetch", wl)
        w, wref = counters(root, "write", wl)
        if not f or not w or "FETCH_SIZE" not in fref or "WRITE_SIZE" not in wref:
            continue
        sf, sw = 524288.0 / fref["FETCH_SIZE"], 524288.0 / wref["WRITE_SIZE"]
        scale_note = "reference copy of the last pass: FETCH_SIZE %.1f KiB, WRITE_SIZE %.1f KiB for 524288 KiB -> factors %.4f, %.4f" % (
            fref["FETCH_SIZE"], wref["WRITE_SIZE"], sf, sw)
        total = 0.0
        for key in f:
            fe = f[key].get("FETCH_SIZE", 0.0)
            wr = w.get(key, {}).get("WRITE_SIZE", 0.0)
            b = (fe * sf + wr * sw) * 1024
            if "calib" not in key[0]:
                total += b
            lines.append("| %s | %s | %d | %.1f | %.1f | %d |" % (wl, key[0], key[1], fe, wr, b))
        traffic[wl] = int(total)
        alg = ALG_BYTES.get(wl)
        lines.append("| %s | **all kernels of a step** | | | | **%d** (algorithmic %s, ratio %s) |" % (
            wl, total, alg if alg else "-", "%.3f" % (total / alg) if alg else "-"))
    with open(os.path.join(ROOT, "profiles", "all_workloads_hbm_traffic_pmc.md"), "w") as fh:
        fh.write("# rocprofv3 --pmc: HBM traffic of every kernel of every bench.py workload (MI355X, gfx950)\n\n"
                 "Two passes per workload W, one counter each:\n\n"
                 "    rocprofv3 --pmc FETCH_SIZE --output-format csv -d " + shown + "/fetch/W -o p -- " + cmd + " --steps 5 --warmup 1 --calibration-copy\n"
                 "    rocprofv3 --pmc WRITE_SIZE --output-format csv -d " + shown + "/write/W -o p -- " + cmd + " --steps 5 --warmup 1 --calibration-copy\n\n"
                 "Each counter is scaled by what it reads for the plain 512 MiB device copy `--calibration-copy` runs first\n"
                 "(" + scale_note + ").\nMeans per dispatch (KiB as the profiler reports them), scaled bytes per launch, and per step the sum over the\n"
                 "workload's kernels against its algorithmic bytes.\n\n"
                 "| workload | kernel | workgroups | FETCH_SIZE KiB | WRITE_SIZE KiB | scaled HBM bytes per launch |\n|---|---|---|---|---|---|\n"
                 + "\n".join(lines) + "\n")
    # ---- SQ counters
    names = ["SQ_INSTS_VALU_MFMA_MOPS_F32", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CYCLES", "SQ_WAVE_CYCLES", "SQ_INSTS_LDS",
             "SQ_LDS_BANK_CONFLICT", "SQ_INSTS_VALU", "SQ_WAIT_INST_ANY", "GRBM_GUI_ACTIVE"]
    lines = []
    per_pair = {}
    calib_listed = False  # the calibration loops run in every pass: their rows are listed once
    for wl in workloads:
        s, _ = counters(root, "sq", wl)
        insts = 0.0
        has_calib = any("calib" in key[0] for key in s)
        for key, v in s.items():
            gui = v.get("GRBM_GUI_ACTIVE", 0.0)
            busy = v.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (1024 * gui / 8) if gui else 0.0
            valu = v.get("SQ_INSTS_VALU", 0.0) * 4 / (1024 * gui / 8) if gui else 0.0
            if "calib" in key[0] and calib_listed:
                continue
            lines.append("| %s | %s | %d | %s | %.3f | %.3f |" % (wl, key[0], key[1], " | ".join("%.4g" % v.get(n, 0.0) for n in names), busy, valu))
            if "calib" not in key[0]:
                insts += v.get("SQ_INSTS_VALU", 0.0)
        calib_listed = calib_listed or has_calib
        if wl in PAIRS:
            per_pair[wl] = round(insts * 64 / PAIRS[wl], 3)
    with open(os.path.join(ROOT, "profiles", "all_workloads_mfma_lds_valu_pmc.md"), "w") as fh:
        fh.write("# rocprofv3 --pmc: MFMA, LDS and VALU counters of every kernel of every bench.py workload (MI355X, gfx950)\n\n"
                 "One pass per workload W (8 SQ counters + 1 GRBM counter):\n\n"
                 "    rocprofv3 --pmc " + " ".join(names) + " --output-format csv -d " + shown + "/sq/W -o p -- " + cmd + " --steps 5 --warmup 1 --valu-kinds\n\n"
                 "Means per dispatch, summed over the chip by the profiler (`--valu-kinds` also runs the calibration loop of every\n"
                 "instruction kind once in every pass; their rows are listed with the first workload only).  The last two columns: MFMA pipe busy = SQ_VALU_MFMA_BUSY_CYCLES / (1024 SIMDs x\n"
                 "GRBM_GUI_ACTIVE / 8 XCDs), and VALU instructions x 4 cycles over the same SIMD cycles -- above 1.0 where the\n"
                 "instruction kinds that issue in about 2 cycles dominate.\n\n"
                 "| workload | kernel | workgroups | " + " | ".join(names) + " | MFMA busy | VALU insts x 4 / SIMD cycles |\n|---|---|---|" + "---|" * (len(names) + 2) + "\n"
                 + "\n".join(lines) + "\n")
    out = {"written_by": "paper_2405_05118_amd/profile_summary.py", "traffic_bytes": traffic, "valu_insts_per_pair": per_pair,
           "kernel_ns_per_step": {k: round(v) for k, v in step_ns.items()}}
    path = os.path.join(HERE, "measured_counters.json")
    old = json.load(open(path)) if os.path.exists(path) else {}
    for k in ("traffic_bytes", "valu_insts_per_pair"):  # keep entries of workloads this run did not cover
        merged = dict(old.get(k, {}))
        merged.update(out[k])
        out[k] = merged
    json.dump(out, open(path, "w"), indent=1, sort_keys=True)
    print("wrote profiles/all_workloads_*.md and", path)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
