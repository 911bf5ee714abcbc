"""Where the time of one tva_tree_verify_attn call goes, from time stamps the kernels take themselves.

A small workload (one sequence, a few thousand cached keys) is a chain of latencies, not a stream of
bytes: launch, the per-sequence scalars, Q, the first K/V tile, the remaining tiles, the stores, the gap
to the merge launch, the merge's own round trip.  The instrumented build of the library
(libtva_timeline.so: the same sources compiled with -DTVA_TIMELINE) records the GPU's constant 100 MHz
clock at those points in every workgroup; this module runs a benchmark workload on it the way bench.py
does (HIP graph over rotating input copies, caches flushed before each replay), reads the stamps of the
last call and prints their distribution over the workgroups.

    python -m paper_2510_26577_amd.timeline --workload cfg2 --out profiles/latency_floor_cfg2.txt

The stamps cost time themselves (a call of the instrumented build is slower than one of libtva.so; both
are printed): read the stages relative to each other.  Only device plumbing and timing live here.
"""
from __future__ import annotations

import argparse
import dataclasses
import sys

import numpy as np

from . import binding, device, workloads

STAGES = ("entry (dispatch skew)", "scalars arrived", "key loop entered (Q, mask rows arrived)", "first tile done",
          "all tiles done", "key groups merged, stores issued")


def get_workload(name: str):
    if name == "cfg1":
        return workloads.config1()
    if name == "cfg2":
        return workloads.config2()
    if name.startswith("cfg2_B"):
        return workloads.config2(int(name[6:]))
    if name.startswith("cfg3_B"):
        return workloads.config3(int(name[6:]))
    if name == "cfg4":
        return workloads.config4()
    raise SystemExit(f"unknown workload {name}")


def per_call_us(lib_is_timeline: bool, w, copies: int, replays: int, num_splits: int, plan_shape: int, cold: bool = True):
    """Times the call (cold caches, HIP graph of `copies` calls) and, on the instrumented build, returns the
    stamps of the last call: (microseconds per call, plan, attention stamps [wgs, 6], merge stamps [blocks, 2])."""
    import torch
    lib = binding.load_library()
    base = device.to_device(w)
    sets = [base] + [dataclasses.replace(base, **{f: getattr(base, f).clone() for f in
                                                  ("q", "k_tree", "v_tree", "k_cache", "v_cache", "parent")})
                     for _ in range(copies - 1)]
    keep, argv = [], []
    for dw in sets:
        out = torch.empty((w.sum_T, w.Hq, w.D), dtype=torch.float32, device="cuda:0")
        lse = torch.empty((w.sum_T, w.Hq), dtype=torch.float32, device="cuda:0")
        args = binding.make_args(q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                                 anc_mask=None, parent=dw.parent, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L,
                                 scale=w.scale, cu_L=dw.cu_L, num_splits=num_splits, out=out, lse=lse,
                                 sum_L=int(w.L.sum()), plan_shape=plan_shape)
        need = binding.workspace_bytes(args)
        ws = torch.empty(max(1, need // 4), dtype=torch.float32, device="cuda:0")
        args.workspace, args.workspace_bytes = ws.data_ptr(), need
        keep.append((out, lse, ws))
        argv.append(args)
    rows, S, ck = binding.plan_workgroup_rows(argv[0]), binding.plan_splits(argv[0]), binding.plan_chunk_keys(argv[0])
    stream = torch.cuda.Stream()
    flush = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0")
    calls = max(len(argv), 64)               # per graph replay: the replay's own launch cost is spread over them
    with torch.cuda.stream(stream):
        for args in argv:
            binding.tree_verify_attn_raw(args, stream=stream)
        stream.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for i in range(calls):
                binding.tree_verify_attn_raw(argv[i % len(argv)], stream=stream)
        for _ in range(3):
            g.replay()
        stream.synchronize()
        ts = []
        for _ in range(replays):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            if cold:
                flush.fill_(1)
            e0.record(stream)
            g.replay()
            e1.record(stream)
            e1.synchronize()
            ts.append(e0.elapsed_time(e1) * 1e3 / calls)
    us = float(np.median(ts))
    if not lib_is_timeline:
        return us, (rows, S, ck), None, None
    G = w.Hq // w.Hkv
    n_wg = w.Hkv * (-(-(w.max_T * G) // rows)) * w.B * S
    n_merge = -(-(w.sum_T * w.Hq) // 4) if S > 1 else 0
    n = min(8192, max(n_wg, n_merge))
    buf = np.zeros((n, 8), dtype=np.uint64)
    rc = lib.tva_timeline_read(buf.ctypes.data, n)
    if rc != 0:
        raise binding.TvaError(rc)
    t = buf.astype(np.int64) * 0.01          # 100 MHz counts -> microseconds
    attn = t[:min(n_wg, n), :6]
    attn = attn[attn[:, 5] > 0]              # (workgroups without rows or keys return early and leave none)
    merge = t[:min(n_merge, n), 6:8]
    return us, (rows, S, ck), attn, merge


def summarise(name, w, us_plain, us_instr, plan, attn, merge, cmd, mode) -> str:
    def st(x):
        return f"min {x.min():6.2f}   median {np.median(x):6.2f}   max {x.max():6.2f}"
    t0 = attn[:, 0].min()
    a = attn - t0
    lines = [
        f"Timeline of one tva_tree_verify_attn call, workload {name} ({w.name}), MI355X",
        f"made by:  {cmd}",
        "(time stamps of the constant 100 MHz clock taken inside the kernels of the instrumented build;",
        " microseconds; distribution over the workgroups of the last call of a HIP-graph replay: " + mode + ")",
        "",
        f"plan: {plan[0]} rows per workgroup, {plan[1]} KV splits of {plan[2]} keys; {len(attn)} attention workgroups"
        + (f", {len(merge)} merge blocks" if merge is not None and len(merge) else ""),
        f"per call, median of the replays: {us_instr:.2f} us (instrumented build)"
        + (f", {us_plain:.2f} us (libtva.so, same protocol)" if us_plain > 0 else ""),
        "",
        "attention kernel, time since the first workgroup's entry:",
        f"  {STAGES[0]:<44s} {st(a[:, 0])}",
    ]
    for i in range(1, 6):
        lines.append(f"  + {STAGES[i]:<42s} {st(a[:, i] - a[:, i - 1])}")
    lines.append(f"  = {'result stores issued, absolute':<42s} {st(a[:, 5])}")
    if merge is not None and len(merge):
        m = merge - t0
        lines += [
            "merge kernel, same clock:",
            f"  {'entry, absolute':<44s} {st(m[:, 0])}",
            f"  + {'partials read, merged, stores issued':<42s} {st(m[:, 1] - m[:, 0])}",
            f"  = {'stores issued, absolute':<42s} {st(m[:, 1])}",
            f"gap between the last attention workgroup's stores and the first merge block: {m[:, 0].min() - a[:, 5].max():.2f} us",
            f"from the first attention entry to the last merge store: {m[:, 1].max():.2f} us; the rest of the "
            f"{us_instr:.2f} us per call is the gap to the next call's first workgroup",
        ]
    else:
        lines.append(f"the rest of the {us_instr:.2f} us per call is the gap to the next call's first workgroup")
    return "\n".join(lines) + "\n"


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--splits", type=int, default=0)
    ap.add_argument("--shape", type=int, default=0)
    ap.add_argument("--copies", type=int, default=64, help="distinct input copies the calls of a replay cycle through")
    ap.add_argument("--warm", action="store_true", help="no cache flush before a replay (with --copies 1: everything "
                                                        "the call touches stays in the caches and the TLBs)")
    ap.add_argument("--replays", type=int, default=5)
    ap.add_argument("--plain-us", type=float, default=0.0,
                    help="per-call time of libtva.so for the same workload (one process loads one build: "
                         "pass the figure of a run with --plain, or of bench.py)")
    ap.add_argument("--plain", action="store_true", help="time libtva.so instead and print microseconds per call")
    ap.add_argument("--out", default="")
    a = ap.parse_args(argv)
    w = get_workload(a.workload)
    if a.plain:
        us, plan, _, _ = per_call_us(False, w, a.copies, a.replays, a.splits, a.shape, cold=not a.warm)
        print(f"{us:.3f}")
        return 0
    binding.use_timeline_library()
    us, plan, attn, merge = per_call_us(True, w, a.copies, a.replays, a.splits, a.shape, cold=not a.warm)
    cmd = "python -m paper_2510_26577_amd.timeline " + " ".join(sys.argv[1:] if argv is None else argv)
    mode = (f"{a.copies} input cop{'y' if a.copies == 1 else 'ies'}, " +
            ("caches left as the calls before leave them" if a.warm else "caches flushed before the replay"))
    text = summarise(a.workload, w, a.plain_us, us, plan, attn, merge, cmd, mode)
    print(text, end="")
    if a.out:
        with open(a.out, "w") as f:
            f.write(text)
    return 0


if __name__ == "__main__":
    sys.exit(main())
