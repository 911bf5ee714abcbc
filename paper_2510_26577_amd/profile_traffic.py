"""HBM traffic of the benchmark's kernels from hardware counters: runs `bench.py` twice under
`rocprofv3 --pmc` (FETCH_SIZE, then WRITE_SIZE: the two do not fit one pass), scales both by what the same
counters read for a plain device-to-device copy of known size made in the same run, and reports bytes per
dispatch of every kernel next to the workload's algorithmic bytes.

    python3 -m paper_2510_26577_amd.profile_traffic cfg2 cfg4 ...     writes profiles/hbm_traffic_<workload>.txt
    python3 bench.py --with-traffic ...                               fills roofline.traffic of that run

Measurement aid: nothing on the hot path imports it.  The profiled program is started directly behind
`rocprofv3 ... --` (python3 bench.py ...), as a child of this process, which itself never touches the GPU."""
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
CAL_KIB = 65536          # bench.py --traffic-probe copies this much once (device to device) for calibration
PROBE = ["--no-cpu-baseline", "--no-saturated", "--steps", "16", "--warmup", "4", "--no-graph", "--traffic-probe"]


def bench_args_of(a) -> list:
    """The workload-defining options of a parsed bench.py command line."""
    out = ["--workload", a.workload]
    if a.splits:
        out += ["--splits", str(a.splits)]
    if a.shape:
        out += ["--shape", str(a.shape)]
    for flag, name in ((a.kv_fp8, "--kv-fp8"), (a.head_major, "--head-major"), (a.no_length_hint, "--no-length-hint")):
        if flag:
            out.append(name)
    return out


def _run(counter: str, bench_args: list, workdir: str):
    d = os.path.join(workdir, counter)
    cmd = ["rocprofv3", "--pmc", counter, "-d", d, "-o", "p", "--output-format", "csv", "--",
           "python3", os.path.join(ROOT, "bench.py"), *bench_args, *PROBE]
    env = dict(os.environ, TMPDIR="/tmp")
    res = subprocess.run(["timeout", "-s", "KILL", "90", *cmd], cwd="/tmp", env=env, stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True)
    if res.returncode != 0:
        raise RuntimeError(f"rocprofv3 --pmc {counter} failed ({res.returncode}):\n{res.stderr[-2000:]}")
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise RuntimeError(f"rocprofv3 --pmc {counter}: no counter_collection.csv under {d}")
    agg = collections.defaultdict(list)
    rows = sorted(csv.DictReader(open(files[0])), key=lambda r: int(r["Dispatch_Id"]))
    cal = None               # the probe's copy is the first plain copy kernel of the run
    for r in rows:
        if cal is None and "copyBuffer" in r["Kernel_Name"]:
            cal = float(r["Counter_Value"])
        agg[(r["Kernel_Name"], r["Grid_Size"])].append(float(r["Counter_Value"]))
    if cal is None:
        raise RuntimeError("no plain copy kernel found for calibration")
    line = next((json.loads(l) for l in res.stdout.splitlines() if l.startswith("{")), None)
    return {k: sum(v) / len(v) for k, v in agg.items()}, cal, line, " ".join(cmd[:-len(PROBE) - len(bench_args) - 2] + ["python3", "bench.py", *bench_args, *PROBE])


def measure(bench_args: list) -> dict:
    work = tempfile.mkdtemp(prefix="tva_traffic_", dir="/tmp")
    try:
        fetch, cal_f, line, cmd_f = _run("FETCH_SIZE", bench_args, work)
        write, cal_w, _, cmd_w = _run("WRITE_SIZE", bench_args, work)
    finally:
        shutil.rmtree(work, ignore_errors=True)
    sf, sw = CAL_KIB / cal_f, CAL_KIB / cal_w
    kernels = {}
    for k, v in fetch.items():
        if "attn_kernel" in k[0] or "merge_kernel" in k[0] or "anc_mask_kernel" in k[0]:
            f_kib, w_kib = v * sf, write.get(k, 0.0) * sw
            kernels[k[0][:96]] = {"fetch_KiB": f_kib, "write_KiB": w_kib, "bytes": (f_kib + w_kib) * 1024}
    attn = max((v["bytes"] for k, v in kernels.items() if "attn_kernel" in k), default=None)
    return {"kernels": kernels, "attn_kernel_bytes": attn, "fetch_scale": sf, "write_scale": sw,
            "calibration_reads": {"FETCH_SIZE": cal_f, "WRITE_SIZE": cal_w}, "bench_line": line,
            "commands": [cmd_f, cmd_w]}


def write_summary(workload: str, t: dict) -> str:
    line = t["bench_line"]
    alg = line["algorithmic_bytes_per_step"]
    out = [f"HBM traffic of the benchmark kernels, workload {workload} ({line['config']['workload']}), rocprofv3 --pmc, MI355X",
           "made by:  python3 -m paper_2510_26577_amd.profile_traffic " + workload, "which runs:"]
    out += ["  " + c for c in t["commands"]]
    out += [f"calibration: the probe's plain device-to-device copy of {CAL_KIB} KiB reads FETCH_SIZE = {t['calibration_reads']['FETCH_SIZE']:.1f}, "
            f"WRITE_SIZE = {t['calibration_reads']['WRITE_SIZE']:.1f}",
            f"             -> scale factors to KiB: {t['fetch_scale']:.4f} (fetch), {t['write_scale']:.4f} (write)", "",
            f"{'kernel (mean per dispatch)':72s} {'fetch_KiB':>12s} {'write_KiB':>12s} {'total_MB':>10s}"]
    for k, v in t["kernels"].items():
        out.append(f"{k[:72]:72s} {v['fetch_KiB']:12.1f} {v['write_KiB']:12.1f} {v['bytes'] / 1e6:10.3f}")
    out += ["", f"algorithmic bytes of one launch (K/V + Q + O + LSE + masks + page table): {alg / 1e6:.3f} MB; kv_splits {line['config']['kv_splits']}",
            f"attention kernel traffic / algorithmic bytes = {t['attn_kernel_bytes'] / alg:.2f}"]
    total = sum(v["bytes"] for k, v in t["kernels"].items() if "attn_kernel" in k or "merge_kernel" in k)
    out.append(f"attention + merge traffic / algorithmic bytes = {total / alg:.2f}")
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload}.txt")
    open(path, "w").write("\n".join(out) + "\n")
    return path


def main(argv):
    for wl in argv or ["cfg1", "cfg2", "cfg2_B32", "cfg3_B1", "cfg3_B4", "cfg3_B16", "cfg3_B64", "cfg4", "cfg5"]:
        t = measure(["--workload", wl])
        print(write_summary(wl, t), f"attention kernel {t['attn_kernel_bytes'] / 1e6:.3f} MB per launch", flush=True)


if __name__ == "__main__":
    main(sys.argv[1:])
