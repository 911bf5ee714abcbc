"""Per-kernel time and wave-level counters of the benchmark's kernels: runs `bench.py` under
`rocprofv3 --kernel-trace --stats` and under three `rocprofv3 --pmc` counter sets, and writes the short
summaries the design document quotes.

    python3 -m paper_2510_26577_amd.profile_kernels trace cfg2 cfg4 ...     profiles/kernel_trace_<workload>.txt
    python3 -m paper_2510_26577_amd.profile_kernels counters cfg2_B32 ...   profiles/counters_<workload>.txt
    python3 -m paper_2510_26577_amd.profile_kernels module draft verify     profiles/kernel_trace_<module>_kernels.txt
                                                                            (the kernels around the attention)

Measurement aid: nothing on the hot path imports it.  The profiled program is started directly behind
`rocprofv3 ... --` (python3 bench.py ...), as a child of this process, which itself never touches the GPU.
A workload name may carry `+fp8` (bench.py --kv-fp8)."""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import shutil
import subprocess
import sys
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
# eager launches, few steps: counters are read per dispatch
PMC_BENCH = ["--no-cpu-baseline", "--no-saturated", "--steps", "8", "--warmup", "2", "--rotate", "2", "--no-graph"]
COUNTER_SETS = (
    ["SQ_BUSY_CU_CYCLES", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_VALU_MFMA_MOPS_BF16", "SQ_INSTS_MFMA", "SQ_INSTS_VALU", "SQ_WAVES",
     "GRBM_GUI_ACTIVE"],
    ["SQ_WAVE_CYCLES", "SQ_BUSY_CYCLES", "SQ_WAIT_ANY", "SQ_WAIT_INST_ANY", "SQ_WAIT_INST_LDS", "SQ_ACTIVE_INST_VALU",
     "SQ_ACTIVE_INST_LDS", "SQ_ACTIVE_INST_VMEM"],
    ["SQ_LDS_BANK_CONFLICT", "SQ_LDS_ADDR_CONFLICT", "SQ_LDS_IDX_ACTIVE", "SQ_LDS_DATA_FIFO_FULL", "SQ_LDS_CMD_FIFO_FULL",
     "SQ_VMEM_TA_ADDR_FIFO_FULL", "SQ_VMEM_TA_CMD_FIFO_FULL", "SQ_VALU_MFMA_COEXEC_CYCLES"],
)


def bench_args(workload: str) -> list:
    name, _, opt = workload.partition("+")
    return ["--workload", name] + (["--kv-fp8"] if opt == "fp8" else [])


def _rocprof(mode_args: list, bargs: list, workdir: str, tag: str):
    d = os.path.join(workdir, tag)
    cmd = ["rocprofv3", *mode_args, "-d", d, "-o", "p", "--output-format", "csv", "--", "python3", os.path.join(ROOT, "bench.py"), *bargs]
    env = dict(os.environ, TMPDIR="/tmp")
    res = subprocess.run(["timeout", "-s", "KILL", "300", *cmd], cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                         text=True)
    if res.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)} failed ({res.returncode}):\n{res.stderr[-2000:]}")
    line = next((json.loads(l) for l in res.stdout.splitlines() if l.startswith("{")), None)
    shown = " ".join(cmd).replace(d, "<dir>").replace(os.path.join(ROOT, "bench.py"), "bench.py")
    return d, line, shown


def trace(workload: str) -> str:
    work = tempfile.mkdtemp(prefix="tva_trace_", dir="/tmp")
    try:
        d, line, shown = _rocprof(["--kernel-trace", "--stats"], bench_args(workload) + ["--no-cpu-baseline", "--no-saturated"], work, "kt")
        files = glob.glob(os.path.join(d, "**", "*kernel_stats.csv"), recursive=True)
        if not files:
            raise RuntimeError("no kernel_stats.csv under " + d)
        rows = list(csv.DictReader(open(files[0])))
    finally:
        shutil.rmtree(work, ignore_errors=True)
    r, t = line["roofline"], line["timing"]
    out = [f"rocprofv3 kernel-trace summary: workload {workload} ({line['config']['workload']}), MI355X (gfx950)",
           "made by:  python3 -m paper_2510_26577_amd.profile_kernels trace " + workload,
           "which runs:  " + shown,
           "(bench.py times five regions -- the one-call step, the attention kernel alone, the attention call, the two-call step,",
           " the merge alone -- each as HIP-graph replays after untimed ones: hence the call counts.  Microseconds; the step times",
           " of a run under the tracer read high.)", "",
           f"{'kernel':72s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'pct':>6s}"]
    for x in rows:
        if float(x["Percentage"]) >= 0.05:
            out.append(f"{x['Name'][:72]:72s} {x['Calls']:>6s} {float(x['AverageNs']) / 1e3:9.3f} {float(x['MinNs']) / 1e3:9.3f} "
                       f"{float(x['MaxNs']) / 1e3:9.3f} {float(x['Percentage']):6.2f}")
    out += ["", "bench.py JSON line of the same (profiled) run:",
            f"  ms_per_step {line['ms_per_step']:.5f} (median; min {t['ms_per_step_min']:.5f})  value {line['value']:.1f} GB/s "
            f"(K/V bytes / step time)  kv_splits {line['config']['kv_splits']}",
            f"  roofline: kernel_ms {r['kernel_ms']:.5f} (attention kernel launched alone in a graph, dispatch gap included); "
            f"whole attention call {r['attn_call_ms']:.5f}; merge alone {r['merge_ms']:.5f}",
            f"            achieved {r['achieved']:.1f} GB/s = frac {r['frac']:.4f} of 8000 GB/s; {r['mfma_tflops']:.1f} TFLOP/s = "
            f"{100 * r['mfma_frac']:.1f}% of 2500"]
    path = os.path.join(ROOT, "profiles", f"kernel_trace_{workload.replace('+', '_')}.txt")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def counters(workload: str) -> str:
    work = tempfile.mkdtemp(prefix="tva_pmc_", dir="/tmp")
    vals, name, cmds = {}, "", []
    try:
        for i, cs in enumerate(COUNTER_SETS):
            d, _, shown = _rocprof(["--pmc", *cs], bench_args(workload) + PMC_BENCH, work, f"set{i}")
            cmds.append(shown)
            files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
            if not files:
                raise RuntimeError("no counter_collection.csv under " + d)
            agg = collections.defaultdict(list)
            for row in csv.DictReader(open(files[0])):
                if "attn_kernel" in row["Kernel_Name"]:
                    name = row["Kernel_Name"]
                    agg[row["Counter_Name"]].append(float(row["Counter_Value"]))
            vals.update({k: sum(v) / len(v) for k, v in agg.items()})
    finally:
        shutil.rmtree(work, ignore_errors=True)
    wc = vals["SQ_WAVE_CYCLES"]
    util = vals["SQ_VALU_MFMA_BUSY_CYCLES"] / (vals["GRBM_GUI_ACTIVE"] / 8 * 1024)
    out = [f"Wave-level counters of the attention kernel, workload {workload}, rocprofv3 --pmc, MI355X",
           "made by:  python3 -m paper_2510_26577_amd.profile_kernels counters " + workload,
           "which runs (one run per counter set; values are sums over the chip, means over the kernel's dispatches):"]
    out += ["  " + c for c in cmds]
    out += ["", "kernel " + name[:110]] + [f"    {k:32s} {v:16.1f}" for k, v in vals.items()]
    out += ["",
            f"MFMA utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs * 1024 SIMDs) = {100 * util:.1f} %",
            f"VALU instructions per MFMA = {vals['SQ_INSTS_VALU'] / max(vals['SQ_INSTS_MFMA'], 1):.1f}",
            f"share of wave time: waiting (s_waitcnt / barrier) {100 * vals['SQ_WAIT_ANY'] / wc:.0f} %, waiting to issue "
            f"{100 * vals['SQ_WAIT_INST_ANY'] / wc:.0f} %, VALU+MFMA issue {100 * vals['SQ_ACTIVE_INST_VALU'] / wc:.0f} %, LDS issue "
            f"{100 * vals['SQ_ACTIVE_INST_LDS'] / wc:.0f} %, vector-memory issue {100 * vals['SQ_ACTIVE_INST_VMEM'] / wc:.0f} %",
            f"LDS bank-conflict cycles / LDS active cycles = {vals['SQ_LDS_BANK_CONFLICT'] / max(vals['SQ_LDS_IDX_ACTIVE'], 1):.2f}",
            f"cycles with MFMA and VALU executing together / MFMA busy cycles = "
            f"{vals['SQ_VALU_MFMA_COEXEC_CYCLES'] / max(vals['SQ_VALU_MFMA_BUSY_CYCLES'], 1):.2f}"]
    path = os.path.join(ROOT, "profiles", f"counters_{workload.replace('+', '_')}.txt")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def module_trace(module: str) -> str:
    """Per-kernel durations of `python3 -m paper_2510_26577_amd.<module>` (the timing programs of the kernels around the
    attention) under rocprofv3 --kernel-trace: one line per kernel and launch shape."""
    if module not in ("draft", "verify"):
        raise ValueError("module: draft or verify")
    work = tempfile.mkdtemp(prefix="tva_mtrace_", dir="/tmp")
    try:
        d = os.path.join(work, "kt")
        cmd = ["rocprofv3", "--kernel-trace", "-d", d, "-o", "p", "--output-format", "csv", "--", "python3", "-m",
               "paper_2510_26577_amd." + module]
        env = dict(os.environ, TMPDIR="/tmp", PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
        res = subprocess.run(["timeout", "-s", "KILL", "600", *cmd], cwd="/tmp", env=env, stdout=subprocess.PIPE, stderr=subprocess.PIPE,
                             text=True)
        if res.returncode != 0:
            raise RuntimeError(f"{' '.join(cmd)} failed ({res.returncode}):\n{res.stderr[-2000:]}")
        files = glob.glob(os.path.join(d, "**", "*kernel_trace.csv"), recursive=True)
        if not files:
            raise RuntimeError("no kernel_trace.csv under " + d)
        agg = collections.defaultdict(list)
        for row in csv.DictReader(open(files[0])):
            name = row["Kernel_Name"]
            if "at::" in name or "elementwise_kernel" in name or "anonymous namespace" not in name:
                continue                                 # (torch's own kernels, which make the inputs, are left out)
            key = (name.replace("(anonymous namespace)::", "").split("(")[0], int(row["Grid_Size_X"]) // max(int(row["Workgroup_Size_X"]), 1),
                   int(row["Grid_Size_Y"]) // max(int(row["Workgroup_Size_Y"]), 1), int(row["Grid_Size_Z"]) // max(int(row["Workgroup_Size_Z"]), 1),
                   int(row["Workgroup_Size_X"]))
            agg[key].append(int(row["End_Timestamp"]) - int(row["Start_Timestamp"]))
    finally:
        shutil.rmtree(work, ignore_errors=True)
    out = [f"rocprofv3 kernel-trace summary of the kernels around the attention: python3 -m paper_2510_26577_amd.{module}, MI355X (gfx950)",
           "made by:  python3 -m paper_2510_26577_amd.profile_kernels module " + module,
           "which runs:  " + " ".join(cmd).replace(d, "<dir>"),
           "(one line per kernel and launch shape, in the order of the program's shapes; microseconds from the tracer's start and end",
           " stamps of each dispatch; the program's own per-call figures, which include the gaps between launches, are in",
           f" profiles/{module}_kernels_timing.txt)", "",
           f"{'kernel':44s} {'workgroups (x, y, z)':>22s} {'threads':>8s} {'calls':>7s} {'median_us':>10s} {'min_us':>8s} {'max_us':>9s}"]
    for (name, gx, gy, gz, wg), v in agg.items():
        v.sort()
        out.append(f"{name[:44]:44s} {f'{gx}, {gy}, {gz}':>22s} {wg:8d} {len(v):7d} {v[len(v) // 2] / 1e3:10.2f} {v[0] / 1e3:8.2f} {v[-1] / 1e3:9.2f}")
    path = os.path.join(ROOT, "profiles", f"kernel_trace_{module}_kernels.txt")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def main(argv) -> int:
    if len(argv) < 2 or argv[0] not in ("trace", "counters", "module"):
        print(__doc__)
        return 2
    for wl in argv[1:]:
        print({"trace": trace, "counters": counters, "module": module_trace}[argv[0]](wl), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
