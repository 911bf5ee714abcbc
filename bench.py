#!/usr/bin/env python3
"""Benchmark of the tree-verification attention hot path on one MI355X.

A step = one pass of the whole path (ancestor sets -> split-KV attention ->
merge) over one batch of seeded synthetic input already resident in HBM, made
as one library call: the trees' parent arrays are passed and the attention
kernel derives each node's ancestor set itself.  The same pass as two calls
(ancestor-mask kernel, then attention on the masks -- what a many-layer model
does once per decode step and once per layer) is timed beside it and reported
as `ms_per_step_two_calls`.  The
default workload is the Llama-3-8B-shaped layer (B=1, Hq=32, Hkv=8, D=128,
L=2048, T=60).  Steps cycle through `rotate` distinct copies of the inputs whose
total size exceeds the last-level cache, and are replayed from one HIP graph so
that host launch overhead is not what is measured (--no-graph: eager launches).

Prints ONE JSON line.  `value` = KV bytes addressed per step / time per step.
`roofline` prices the dominant kernel (the split-KV attention kernel) against
the HBM peak using the algorithmic bytes of one launch; `cpu_baseline` is the
CPU oracle timed on this machine's host cores on the same workload.  With the
default workload, `roofline_saturating_batch` holds the same kernel-level
figures for the same shape at B=32 (--no-saturated skips it).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0


def get_workload(name):
    from paper_2510_26577_amd import workloads as wl
    if name == "cfg1":
        return wl.config1()
    if name == "cfg2":
        return wl.config2()
    if name.startswith("cfg2_B"):
        return wl.config2(int(name[6:]))
    if name.startswith("cfg3_B"):
        return wl.config3(int(name[6:]))
    if name == "cfg4":
        return wl.config4()
    if name == "cfg5":
        return wl.config5()
    if name.startswith("custom:"):
        # custom:B=32,Hq=32,Hkv=8,D=128,L=2048,T=60[,page=16]  (uniform L and T, random trees of depth <= 8)
        kv = dict(item.split("=") for item in name[7:].split(","))
        g = lambda k, d: int(kv.get(k, d))
        return wl.random_workload(12345, g("B", 1), g("Hq", 32), g("Hkv", 8), g("D", 128), g("L", 2048), g("T", 60),
                                  max_depth=8, page_size=g("page", 0), name=name)
    raise SystemExit(f"unknown workload {name}")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=32)
    ap.add_argument("--workload", default="cfg2")
    ap.add_argument("--splits", type=int, default=0, help="KV splits (0 = library chooses)")
    ap.add_argument("--shape", type=int, default=0, help="workgroup shape (tva_shape 1..5; 0 = library chooses)")
    ap.add_argument("--rotate", type=int, default=0, help="distinct input copies (0 = enough to exceed 640 MB)")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--head-major", action="store_true",
                    help="store the dense cache as [Hkv, sum_L, D] (passed through the stride arguments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-saturated", action="store_true",
                    help="default workload only: skip the extra kernel-level measurement of the same shape at B=32")
    ap.add_argument("--no-length-hint", action="store_true",
                    help="do not pass the host-known cache lengths (their sum: launch planner; the lengths: which "
                         "sequences share a CU) to the library")
    ap.add_argument("--reps", type=int, default=5, help="timed replays per figure (median and minimum are reported)")
    ap.add_argument("--with-traffic", action="store_true",
                    help="also measure roofline.traffic: two child runs of this command under rocprofv3 --pmc "
                         "(the full default run, with the CPU baseline, does so anyway)")
    ap.add_argument("--no-traffic", action="store_true", help="leave roofline.traffic null")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="(used by profile_traffic) make one plain 64 MiB device-to-device copy first: the counters' calibration")
    ap.add_argument("--microbench", action="store_true",
                    help="run the microbenchmarks of the machine rates (libtva_ubench) instead of a workload")
    ap.add_argument("--kv-fp8", action="store_true",
                    help="K/V stored as 8-bit floating point (E4M3) bytes: half the K/V bytes per step")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        raise SystemExit(2)
    if a.microbench:
        from paper_2510_26577_amd import ubench
        print(json.dumps({"microbench": ubench.run_all(), "device": "MI355X (gfx950)", "n_gpus": 1}))
        return
    line = measure(a)
    if a.workload == "cfg2" and not (a.kv_fp8 or a.head_major or a.no_graph or a.splits or a.shape or a.no_saturated):
        # The headline shape at B = 1 is ~1 us of HBM time: its roofline fraction mostly measures launch
        # latency.  The same shape at a batch that fills the chip is measured beside it (kernel-level figures
        # only; `value` stays the B = 1 step).
        import copy
        import torch
        torch.cuda.empty_cache()
        b = copy.copy(a)
        b.workload, b.steps, b.warmup, b.no_cpu_baseline = "cfg2_B32", min(a.steps, 64), 8, True
        sat = measure(b)
        line["roofline_saturating_batch"] = dict(sat["roofline"], workload=sat["config"]["workload"], B=sat["config"]["B"],
                                                 ms_per_step=sat["ms_per_step"], kv_gbs=sat["value"], steps=b.steps)
    print(json.dumps(line))


def measure(a):
    """One workload: builds the inputs, times the step and the kernels, returns the result line as a dict."""
    import numpy as np
    import torch
    from paper_2510_26577_amd import binding, device

    binding.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if a.traffic_probe:
        cal_src = torch.ones(1 << 24, dtype=torch.int32, device="cuda:0")      # 64 MiB
        cal_dst = torch.empty_like(cal_src)
        cal_dst.copy_(cal_src)
        torch.cuda.synchronize()
        del cal_src, cal_dst
    w = get_workload(a.workload)
    k_scale = v_scale = 1.0
    if a.kv_fp8:
        from paper_2510_26577_amd import workloads as wl
        w, k_scale, v_scale = wl.to_fp8_kv(w)
    sum_L = 0 if a.no_length_hint else int(w.L.sum())   # the serving side knows its sequence lengths
    L_host = None if a.no_length_hint else np.ascontiguousarray(w.L, dtype=np.int32)
    kv_bytes, alg_bytes, flops = w.kv_bytes(), w.algorithmic_bytes(), w.algorithmic_flops()
    R = a.rotate or max(2, min(64, -(-640 * 2 ** 20 // alg_bytes)))

    # ---- inputs: one seeded set, R-1 device copies at distinct addresses ----
    base = device.to_device(w)
    strides = (0, 0, 0)
    if a.head_major and not w.paged:
        base.k_cache = base.k_cache.permute(1, 0, 2).contiguous()
        base.v_cache = base.v_cache.permute(1, 0, 2).contiguous()
        strides = (0, w.D, int(w.L.sum()) * w.D)
    sets = [base]
    import dataclasses
    for _ in range(R - 1):
        sets.append(dataclasses.replace(base, **{f: getattr(base, f).clone() for f in
                                                ("q", "k_tree", "v_tree", "k_cache", "v_cache", "parent")}))
    masks = [torch.empty((w.sum_T, max(1, (w.max_T + 63) // 64)), dtype=torch.int64, device="cuda:0") for _ in sets]
    outs = [torch.empty((w.sum_T, w.Hq, w.D), dtype=torch.float32, device="cuda:0") for _ in sets]
    lses = [torch.empty((w.sum_T, w.Hq), dtype=torch.float32, device="cuda:0") for _ in sets]
    argv = []
    for dw, m, o, l in zip(sets, masks, outs, lses):
        args = binding.make_args(q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                                 anc_mask=m, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L, scale=w.scale,
                                 cu_L=dw.cu_L, page_table=dw.page_table, page_size=w.page_size,
                                 strides=strides, num_splits=a.splits, out=o, lse=l, kv_fp8=a.kv_fp8, k_scale=k_scale,
                                 v_scale=v_scale, sum_L=sum_L, plan_shape=a.shape, L_host=L_host)
        argv.append(args)
    # the same calls with the parent arrays in place of ancestor masks (the kernel derives the masks)
    argv_parent = []
    for dw, o, l in zip(sets, outs, lses):
        argv_parent.append(binding.make_args(
            q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache, anc_mask=None,
            parent=dw.parent, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L, scale=w.scale, cu_L=dw.cu_L,
            page_table=dw.page_table, page_size=w.page_size, strides=strides, num_splits=a.splits, out=o, lse=l,
            kv_fp8=a.kv_fp8, k_scale=k_scale, v_scale=v_scale, sum_L=sum_L, plan_shape=a.shape, L_host=L_host))
    n_splits = binding.plan_splits(argv[0])
    ws_bytes = binding.workspace_bytes(argv[0])
    wss = []
    for args, args_p in zip(argv, argv_parent):
        if ws_bytes:
            ws = torch.empty(ws_bytes // 4, dtype=torch.float32, device="cuda:0")
            wss.append(ws)
            args.workspace, args.workspace_bytes = ws.data_ptr(), ws_bytes
            args_p.workspace, args_p.workspace_bytes = ws.data_ptr(), ws_bytes

    stream = torch.cuda.Stream()   # default priority; all launches and events use this stream

    def step(i):
        """One pass of the whole path as ONE call: the parent arrays are passed and the attention
        kernel derives the ancestor sets itself (then the merge of the KV splits)."""
        binding.tree_verify_attn_raw(argv_parent[i % R], stream=stream)

    def step_two_calls(i, with_mask=True):
        """The same path as two calls: the ancestor-mask kernel, then attention reading the masks
        (what a model with many layers does: masks once per decode step, attention per layer)."""
        j = i % R
        if with_mask:
            binding.build_ancestor_mask(sets[j].parent, sets[j].cu_T, w.max_T, mask=masks[j], stream=stream)
        binding.tree_verify_attn_raw(argv[j], stream=stream)

    # a buffer four times the 256 MB last-level cache: writing it between timed regions evicts whatever the
    # region before (or the warm-up) left in the caches, so a timed region reads its inputs from HBM
    # however few of the rotating copies it touches
    flush_buf = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0")
    REPS = 1 if a.no_graph else max(1, a.reps)

    def timed(n, fn, cold=True):
        """Runs fn(i) for i < n on `stream` as one HIP-graph replay (eager with --no-graph), REPS times,
        each preceded (cold) by the cache flush; returns the REPS durations in ms per call of fn."""
        if a.no_graph:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                e0.record(stream)
                for i in range(n):
                    fn(i)
                e1.record(stream)
            torch.cuda.synchronize()
            return [e0.elapsed_time(e1) / n]
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for i in range(n):
                fn(i)
        out = []
        with torch.cuda.stream(stream):
            # untimed replays first (graph upload, then enough work for the clocks to settle under
            # this load: the first region timed after the host-side set-up otherwise reads ~7 % slow
            # on the large workloads), then the timed ones
            t_warm = time.perf_counter()
            while True:
                g.replay()
                torch.cuda.synchronize()
                if time.perf_counter() - t_warm > 0.1:
                    break
            for _ in range(REPS):
                if cold:
                    flush_buf.fill_(1)
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                torch.cuda.synchronize()
                out.append(e0.elapsed_time(e1) / n)
        return out

    def med(xs):
        xs = sorted(xs)
        return xs[len(xs) // 2] if len(xs) % 2 else 0.5 * (xs[len(xs) // 2 - 1] + xs[len(xs) // 2])

    # ---- warm-up (eager: also raises the LDS limit of the kernels before any capture) ----
    with torch.cuda.stream(stream):
        for i in range(max(a.warmup, R)):
            step(i)
            step_two_calls(i)
    torch.cuda.synchronize()

    # ---- the timed region: exactly K steps of the whole path (one graph replay), REPS times, each
    #      starting from flushed caches; `ms_per_step` is the median, the minimum is reported beside it ----
    step_runs = timed(a.steps, step)
    ms_step, ms_step_min = med(step_runs), min(step_runs)
    # the same with every step on ONE input set and no flush (inputs cache-resident), and one isolated step
    ms_step_warm = med(timed(a.steps, lambda i: step(0), cold=False))
    single = timed(1, lambda i: step(0), cold=True) if not a.no_graph else [ms_step]
    ms_single_launch = med(single)

    # ---- dominant kernel: K launches of the split-KV attention kernel alone (same graph replay,
    #      same rotation; the average includes the dispatch gap between back-to-back launches),
    #      and the merge kernel alone the same way ----
    kernel_runs = timed(a.steps, lambda i: binding.tree_verify_attn_splits_raw(argv[i % R], stream=stream))
    ms_kernel, ms_kernel_min = med(kernel_runs), min(kernel_runs)
    ms_attn_call = med(timed(a.steps, lambda i: step_two_calls(i, with_mask=False)))
    ms_step_two_calls = med(timed(a.steps, step_two_calls))
    ms_merge = 0.0
    if n_splits > 1:
        n_rows = w.sum_T * w.Hq
        po = [ws[: n_splits * n_rows * w.D].view(n_splits, n_rows, w.D) for ws in wss]
        pl = [ws[n_splits * n_rows * w.D: n_splits * n_rows * (w.D + 1)].view(n_splits, n_rows) for ws in wss]
        ms_merge = med(timed(a.steps, lambda i: binding.merge_splits(po[i % R], pl[i % R], out=outs[i % R].view(n_rows, w.D),
                                                                     lse=lses[i % R].view(n_rows), stream=stream)))

    # ---- the CPU oracle leg (--no-cpu-baseline skips all of it; nothing else here touches the oracle):
    # first a spot check of what was just timed (first input set, sampled rows), then the oracle timed on
    # the same workload as the reported baseline (not a target) ----
    cpu = None
    err_o = err_l = None
    if not a.no_cpu_baseline:
        from oracle import tva_oracle
        if a.kv_fp8:
            from oracle import fp8_oracle
            oracle_attn = lambda rows=None: fp8_oracle.tree_verify_attn_fp8(w, k_scale, v_scale, rows=rows)
        else:
            oracle_attn = lambda rows=None: tva_oracle.tree_verify_attn(w, rows=rows) if rows is not None \
                else tva_oracle.tree_verify_attn(w)
        rng = np.random.Generator(np.random.PCG64(7))
        rows = [(b, int(rng.integers(0, w.T[b])), int(rng.integers(0, w.Hq))) for b in rng.integers(0, w.B, size=8)]
        ro, rl = oracle_attn(rows)
        o0, l0 = outs[0].cpu().numpy(), lses[0].cpu().numpy()
        err_o = max(float(np.abs(o0[w.cu_T[b] + i, h] - ro[n]).max()) for n, (b, i, h) in enumerate(rows))
        err_l = max(float(abs(l0[w.cu_T[b] + i, h] - rl[n])) for n, (b, i, h) in enumerate(rows))
        assert err_o <= 2e-3 and err_l <= 1e-4, (err_o, err_l)
        cores = tva_oracle.num_threads()
        full_s = None
        t0 = time.perf_counter()
        if flops <= 8e9:                       # whole workload, best of up to 3 runs within ~20 s
            best = 1e30
            for _ in range(3):
                t1 = time.perf_counter()
                oracle_attn()
                best = min(best, time.perf_counter() - t1)
                if time.perf_counter() - t0 > 20:
                    break
            full_s, sample = best, "whole workload, best of 3 runs"
        else:                                  # bounded sample of output rows, scaled to the whole workload
            n_rows_total = w.sum_T * w.Hq
            n_s = max(cores * 4, int(n_rows_total * 4e9 / flops))
            srows = [(b, int(rng.integers(0, w.T[b])), int(rng.integers(0, w.Hq)))
                     for b in rng.integers(0, w.B, size=n_s)]
            t1 = time.perf_counter()
            oracle_attn(srows)
            dt = time.perf_counter() - t1
            f_s = sum(4 * w.D * (int(w.L[b]) + int(w.T[b])) for b, _, _ in srows)
            full_s, sample = dt * flops / f_s, f"{n_s} random output rows of {n_rows_total}, time scaled by flops"
        cpu = {"value": kv_bytes / full_s / 1e9, "unit": "GB/s", "cores": cores, "kind": "oracle",
               "sample": sample, "ms_per_step": full_s * 1e3}
        if flops <= 8e9:                       # small workloads (configs 1-2): the same on one host thread
            tva_oracle.set_num_threads(1)
            t1 = time.perf_counter()
            oracle_attn()
            one_s = time.perf_counter() - t1
            tva_oracle.set_num_threads(cores)
            cpu["one_thread"] = {"value": kv_bytes / one_s / 1e9, "unit": "GB/s", "cores": 1, "ms_per_step": one_s * 1e3}

    # HBM bytes per launch of the dominant kernel: only from a counter run made for this very command (two child
    # runs of this script under rocprofv3 --pmc, after the timed regions); otherwise null.  The full run (the one
    # with the CPU baseline) makes them; the short forms only with --with-traffic.
    traffic, traffic_note = None, None
    if a.with_traffic or not (a.no_traffic or a.no_cpu_baseline or a.traffic_probe):
        from paper_2510_26577_amd import profile_traffic
        try:
            t = profile_traffic.measure(profile_traffic.bench_args_of(a))
            traffic = t["attn_kernel_bytes"]
            traffic_note = (f"FETCH_SIZE x {t['fetch_scale']:.3f} + WRITE_SIZE x {t['write_scale']:.3f} KiB per dispatch "
                            f"(scales from a 64 MiB copy in the same runs)")
        except Exception as e:  # the counters are evidence beside the timing, never a reason to lose the line
            traffic_note = "not measured: " + str(e).splitlines()[0][:200]
    value = kv_bytes / (ms_step * 1e-3) / 1e9
    achieved = alg_bytes / (ms_kernel * 1e-3) / 1e9
    tflops_kernel = flops / (ms_kernel * 1e-3) / 1e12
    line = {
        "metric": "tree-verify attention: KV GB/s and TFLOP/s (% of MI355X peak), 8B shape",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D,
                   "L": [int(w.L.min()), int(w.L.max())], "T": int(w.max_T), "paged": bool(w.paged), "kv_storage": "e4m3" if a.kv_fp8 else "bf16",
                   "kv_splits": n_splits, "workgroup_rows": binding.plan_workgroup_rows(argv[0]),
                   "host_lengths_given": not a.no_length_hint,
                   "split_keys": binding.plan_chunk_keys(argv[0]), "rotating_input_copies": R, "launch": "eager" if a.no_graph else "hip-graph",
                   "step": "one tva_tree_verify_attn call on parent arrays (ancestor sets derived in the kernel) "
                           "incl. merge of the KV splits; ms_per_step_two_calls = mask kernel + attention on masks"},
        "tflops": flops / (ms_step * 1e-3) / 1e12,
        "pct_hbm_peak": 100 * value / HBM_PEAK_GBS,
        "pct_mfma_peak": 100 * flops / (ms_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
        "kv_bytes_per_step": kv_bytes, "algorithmic_bytes_per_step": alg_bytes, "algorithmic_flops_per_step": flops,
        "max_abs_err_O": err_o, "max_abs_err_LSE": err_l,
        "ms_per_step_two_calls": ms_step_two_calls,
        "timing": {"protocol": f"{REPS} timed replays of one HIP graph of {a.steps} steps cycling through "
                               f"{R} input copies ({R * alg_bytes / 2**20:.0f} MiB), caches flushed by a 1 GiB fill before each; "
                               "ms_per_step = median",
                   "ms_per_step_median": ms_step, "ms_per_step_min": ms_step_min,
                   "ms_per_step_warm_one_input_set": ms_step_warm, "ms_single_isolated_step": ms_single_launch,
                   "kernel_ms_median": ms_kernel, "kernel_ms_min": ms_kernel_min, "reps": REPS},
        "roofline": {"bound": "hbm", "kernel": "attn_kernel (split-KV attention)", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "traffic_note": traffic_note,
                     "kernel_ms": ms_kernel, "attn_call_ms": ms_attn_call, "merge_ms": ms_merge,
                     "mfma_tflops": tflops_kernel, "mfma_frac": tflops_kernel / MFMA_BF16_PEAK_TFLOPS},
        "cpu_baseline": cpu,
    }
    return line


if __name__ == "__main__":
    main()
