"""Few query rows per KV head: the 32-row matrix-instruction shape of libtva against an alternative on the
vector ALUs, by time and by hardware counters.

With T tree tokens and G query heads per KV head a workgroup sees T * G query rows; the smallest shape of
tva_tree_verify_attn pads them to 32 rows of v_mfma_f32_32x32x16_bf16.  Whether that padding costs anything
is an empirical question on three shapes where the rows are few:

    cfg1        benchmark configuration 1: B = 1, Hq = Hkv = 4, D = 64, L = 128, T = 8            8 rows
    decode_B64  plain decoding as a tree of one node: B = 64, Hq 32, Hkv 8, D 128, L ~ U{512..2048}   4 rows
    draft_q12   draft-stage attention (paper, "Dynamic Expansion Stage": the newest layer of the tree attends
                to the cache and the layers before it): B = 8, Hq 16, Hkv 8, D 128, L = 1024, trees of 36
                nodes of which the last 12 are queries                                            24 rows

The alternative is tva_ubench_valu_attn (include/tva_ubench.h), a kernel of the measurement library, not of the
product.  Both are run on the same seeded inputs; their outputs must agree to the parity tolerance.

    python3 -m paper_2510_26577_amd.small_rows                 writes profiles/small_rows_mfma_vs_valu.txt

Timing: HIP graph over 8 input copies, caches flushed before each of 5 replays, median.  Counters: this
module starts itself twice under `rocprofv3 --pmc` (--probe CASE runs a few eager launches of both kernels),
once for the instruction counters, once for FETCH_SIZE.  Only device plumbing and timing live here.
"""
from __future__ import annotations

import argparse
import collections
import csv
import ctypes
import glob
import os
import shutil
import subprocess
import sys
import tempfile

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CASES = ("cfg1", "decode_B64", "draft_q12")
SQ_COUNTERS = ["SQ_INSTS_VALU", "SQ_INSTS_MFMA", "SQ_VALU_MFMA_BUSY_CYCLES", "SQ_INSTS_LDS", "SQ_BUSY_CU_CYCLES"]
TOL_O, TOL_LSE = 2e-3, 1e-4
# measured on this chip (profiles/microbench_mi355x.txt): streaming read rate of LDS-writing loads, and the cost of
# an empty launch inside a graph; bytes / rate + launch is what no kernel for the shape can beat
STREAM_TBS, LAUNCH_US = 5.2, 1.6


class AttnArgs(ctypes.Structure):
    """Mirror of tva_ubench_attn_args."""
    _fields_ = [(n, ctypes.c_void_p) for n in ("q", "k_cache", "v_cache", "k_tree", "v_tree", "mask", "cu_T", "L", "cu_L", "cu_Q")] + \
               [(n, ctypes.c_int32) for n in ("B", "Hq", "Hkv", "D", "mask_words", "max_rows")] + \
               [("scale", ctypes.c_float), ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p)]


def make_case(name: str, seed: int = 0):
    """Returns (workload, query nodes per sequence or None)."""
    from . import workloads
    if name == "cfg1":
        return workloads.config1(), None
    rng = np.random.Generator(np.random.PCG64(2510 + seed))
    if name == "decode_B64":
        L = rng.integers(512, 2049, size=64)
        return workloads.random_workload(71 + seed, 64, 32, 8, 128, L, [1] * 64, name=name), None
    if name == "draft_q12":
        return workloads.random_workload(72 + seed, 8, 16, 8, 128, [1024] * 8, [36] * 8, max_depth=6, name=name), 12
    raise SystemExit(f"unknown case {name}")


class Prepared:
    """Device tensors and the argument blocks of both kernels for one input copy."""

    def __init__(self, name: str, seed: int):
        import torch
        from . import binding, device
        w, nq = make_case(name, seed)
        dw = device.to_device(w)
        self.w, self.dw = w, dw
        self.mask = device.build_mask(dw)
        G = w.Hq // w.Hkv
        if nq is None:
            q, cu_Q, max_Q, self.rows = dw.q, None, 0, int(w.max_T) * G
        else:
            idx = np.concatenate([np.arange(w.cu_T[b + 1] - nq, w.cu_T[b + 1]) for b in range(w.B)])
            q = dw.q[torch.from_numpy(idx).to(dw.q.device)].contiguous()
            cu_Q = torch.from_numpy((np.arange(w.B + 1) * nq).astype(np.int32)).to(dw.q.device)
            max_Q, self.rows = nq, nq * G
        self.q, self.cu_Q = q, cu_Q
        mk = lambda: (torch.empty(q.shape, dtype=torch.float32, device=q.device),
                      torch.empty(q.shape[:2], dtype=torch.float32, device=q.device))
        self.out_m, self.lse_m = mk()
        self.out_v, self.lse_v = mk()
        self.args = binding.make_args(q=q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                                      anc_mask=self.mask, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L, scale=w.scale,
                                      cu_L=dw.cu_L, out=self.out_m, lse=self.lse_m, cu_Q=cu_Q, max_Q=max_Q,
                                      sum_L=int(w.L.sum()))
        need = binding.workspace_bytes(self.args)
        self.ws = torch.empty(max(1, need // 4), dtype=torch.float32, device=q.device)
        self.args.workspace, self.args.workspace_bytes = self.ws.data_ptr(), need
        self.plan = (binding.plan_workgroup_rows(self.args), binding.plan_splits(self.args))
        a = AttnArgs()
        a.q, a.k_cache, a.v_cache = q.data_ptr(), dw.k_cache.data_ptr(), dw.v_cache.data_ptr()
        a.k_tree, a.v_tree, a.mask = dw.k_tree.data_ptr(), dw.v_tree.data_ptr(), self.mask.data_ptr()
        a.cu_T, a.L, a.cu_L = dw.cu_T.data_ptr(), dw.L.data_ptr(), dw.cu_L.data_ptr()
        a.cu_Q = cu_Q.data_ptr() if cu_Q is not None else None
        a.B, a.Hq, a.Hkv, a.D, a.mask_words, a.max_rows = w.B, w.Hq, w.Hkv, w.D, int(self.mask.shape[1]), self.rows
        a.scale, a.out, a.lse = float(w.scale), self.out_v.data_ptr(), self.lse_v.data_ptr()
        self.valu_args = a

    def run_mfma(self, stream):
        from . import binding
        binding.tree_verify_attn_raw(self.args, stream=stream)

    def run_valu(self, stream):
        from . import ubench
        rc = ubench.load_library().tva_ubench_valu_attn(ctypes.byref(self.valu_args), ctypes.c_void_p(stream.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"tva_ubench_valu_attn returned {rc}")


def time_case(name: str, copies: int = 8, replays: int = 5):
    """Microseconds per call of both kernels, their largest difference, and the plan of the product path."""
    import torch
    sets = [Prepared(name, k) for k in range(copies)]
    stream = torch.cuda.Stream()
    flush = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0")
    res = {}
    with torch.cuda.stream(stream):
        for which in ("mfma", "valu"):
            fn = (lambda s: s.run_mfma(stream)) if which == "mfma" else (lambda s: s.run_valu(stream))
            for s in sets:
                fn(s)
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for s in sets:
                    fn(s)
            for _ in range(3):
                g.replay()
            stream.synchronize()
            ts = []
            for _ in range(replays):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                flush.fill_(1)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / len(sets))
            res[which] = float(np.median(ts))
    s = sets[0]
    d_o = float((s.out_m - s.out_v).abs().max())
    fin = torch.isfinite(s.lse_m)
    d_l = float((s.lse_m[fin] - s.lse_v[fin]).abs().max()) if bool(fin.any()) else 0.0
    assert bool((torch.isfinite(s.lse_v) == fin).all())
    return res, (d_o, d_l), s.plan, s.rows, s.w


def probe(name: str) -> None:
    """A few eager launches of both kernels: what the counter runs profile."""
    import torch
    s = Prepared(name, 0)
    st = torch.cuda.current_stream()
    for _ in range(4):
        s.run_mfma(st)
        s.run_valu(st)
    torch.cuda.synchronize()


def counters(name: str, counter_list, workdir: str):
    """Mean counter values per dispatch, by kernel: {kernel: {counter: value}}, and the command."""
    d = os.path.join(workdir, name + "_" + counter_list[0])
    cmd = ["rocprofv3", "--pmc", *counter_list, "-d", d, "-o", "p", "--output-format", "csv", "--",
           "python3", "-m", "paper_2510_26577_amd.small_rows", "--probe", name]
    env = dict(os.environ, TMPDIR="/tmp", PYTHONPATH=ROOT + os.pathsep + os.environ.get("PYTHONPATH", ""))
    r = subprocess.run(["timeout", "-s", "KILL", "180", *cmd], cwd="/tmp", env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.PIPE, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"{' '.join(cmd)} failed ({r.returncode}):\n{r.stderr[-2000:]}")
    files = glob.glob(os.path.join(d, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        raise RuntimeError("no counter_collection.csv under " + d)
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for row in csv.DictReader(open(files[0])):
        k = row["Kernel_Name"]
        kind = "valu" if "valu_attn_kernel" in k else "mfma" if "attn_kernel" in k else "merge" if "merge_kernel" in k else None
        if kind:
            agg[kind][row["Counter_Name"]].append(float(row["Counter_Value"]))
    shown = " ".join(cmd).replace(d, "<dir>")
    return {k: {c: float(np.mean(v)) for c, v in cs.items()} for k, cs in agg.items()}, shown


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--probe", default="", help="run a few launches of both kernels on this case and exit")
    ap.add_argument("--no-counters", action="store_true")
    ap.add_argument("--out", default=os.path.join(ROOT, "profiles", "small_rows_mfma_vs_valu.txt"))
    a = ap.parse_args(argv)
    if a.probe:
        probe(a.probe)
        return 0
    # counters first: the children use the GPU one at a time, before this process touches it
    cnt, cmds = {}, []
    if not a.no_counters:
        work = tempfile.mkdtemp(prefix="tva_small_rows_", dir="/tmp")
        try:
            for name in CASES:
                c1, cmd1 = counters(name, SQ_COUNTERS, work)
                c2, cmd2 = counters(name, ["FETCH_SIZE"], work)
                for k in c1:
                    c1[k].update(c2.get(k, {}))
                cnt[name] = c1
                cmds += [cmd1, cmd2]
        finally:
            shutil.rmtree(work, ignore_errors=True)
    lines = ["Few query rows per KV head: 32-row matrix-instruction shape (libtva) against attention on the vector ALUs",
             "(tva_ubench_valu_attn), MI355X", "made by:  python3 -m paper_2510_26577_amd.small_rows", "which runs:"]
    lines += ["  " + c for c in cmds[:2]] + (["  (the same two for the other cases)"] if cmds else [])
    lines += ["", f"{'case':12s} {'rows':>4s} {'kernel':28s} {'us/call':>8s} {'floor us':>8s} {'VALU insts':>11s} {'MFMA insts':>11s} "
                  f"{'MFMA busy cyc':>13s} {'LDS insts':>10s} {'FETCH KiB*':>10s}   max|dO| max|dLSE|"]
    for name in CASES:
        t, (d_o, d_l), plan, rows, w = time_case(name)
        assert d_o <= TOL_O and d_l <= TOL_LSE, (name, d_o, d_l)
        c = cnt.get(name, {})
        floor = w.algorithmic_bytes() / (STREAM_TBS * 1e6) + LAUNCH_US

        def row(kind, label, us):
            v = c.get(kind, {})
            g = lambda k: f"{v[k]:.0f}" if k in v else "-"
            return (f"{name:12s} {rows:4d} {label:28s} {us:8.2f} {floor:8.2f} {g('SQ_INSTS_VALU'):>11s} {g('SQ_INSTS_MFMA'):>11s} "
                    f"{g('SQ_VALU_MFMA_BUSY_CYCLES'):>13s} {g('SQ_INSTS_LDS'):>10s} {g('FETCH_SIZE'):>10s}")
        lines.append(row("mfma", f"libtva {plan[0]}-row shape, S={plan[1]}", t["mfma"]) + f"   {d_o:.1e} {d_l:.1e}")
        if plan[1] > 1:
            lines.append(row("merge", "  (its merge kernel)", float("nan")))
        lines.append(row("valu", "vector-ALU alternative", t["valu"]))
        print(lines[-1], flush=True)
    lines += ["", "us/call: whole call (libtva: attention + merge of the KV splits), median of 5 cold HIP-graph replays over 8 input copies.",
              f"floor us: the workload's algorithmic bytes at the measured streaming rate ({STREAM_TBS} TB/s) plus one empty launch ({LAUNCH_US} us):",
              "what remains for ANY alternative kernel to gain is us/call minus this.",
              "Counters: mean per dispatch over the launches of a short eager run; instruction counts are per wave-instruction,",
              "FETCH KiB* is the raw counter (about half the KiB actually fetched on this chip, see profiles/hbm_traffic_*.txt).",
              "max|dO|, max|dLSE|: largest difference between the two kernels' outputs on the first input copy."]
    text = "\n".join(lines) + "\n"
    print(text, end="")
    with open(a.out, "w") as f:
        f.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
