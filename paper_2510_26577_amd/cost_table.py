"""Measures the attention part of the target-model cost table S_T(B) on the GPU.

The tree builder (include/tva_cast.h) prices one more verified token with a lookup table
f_T(B, c, n) kept for contexts c = L, 2L, .., M*L and n = 1..N tree tokens (paper, section
"Method").  This module fills the attention slice of that table by timing this library's own
tva_tree_verify_attn (split-KV attention + merge of the splits) at every grid point, on seeded
synthetic inputs of the benchmark's head shapes.  The rest of a target forward (projections, MLP)
is outside this repository; a deployment adds its own measurements of those to the table.

Timing: per grid point, R copies of the inputs, their attention calls captured into one HIP graph,
the graph replayed a few times with the caches flushed before each replay (every call reads its K/V
from HBM, as a layer of a real verification pass does); the cost is the median replay divided by R,
in microseconds.

    python -m paper_2510_26577_amd.cost_table --B 4 --L 256 --M 8 --N 72 --out table.txt

Only device plumbing and timing live here; all arithmetic runs in libtva.so.
"""
from __future__ import annotations

import argparse
import dataclasses
import sys
import time

import numpy as np

from . import binding, device, workloads


def measure(B: int, L: int, M: int, N: int, Hq: int = 32, Hkv: int = 8, D: int = 128, copies: int = 8,
            replays: int = 7, n_values=None, seed: int = 2510, log=None) -> np.ndarray:
    """Returns a float64 [M, N] table of microseconds per attention call; entries for n not in
    n_values (default: all of 1..N) are filled by linear interpolation between measured ones."""
    import torch
    assert torch.cuda.is_available(), "the cost table is measured on the GPU"
    binding.load_library()
    n_values = sorted(set(n_values or range(1, N + 1)) | {1, N})
    table = np.full((M, N), np.nan)
    stream = torch.cuda.Stream()
    # written before every timed replay: four times the 256 MB last-level cache, so every call of the replay
    # reads its inputs from HBM, as a layer of a real verification pass does
    flush = torch.empty(1 << 28, dtype=torch.int32, device="cuda:0")
    for r in range(1, M + 1):
        c = r * L
        # one cache and one N-node tree per copy; the n-token cases use the tree's first n nodes
        # (a prefix of a topologically ordered parent array is a tree)
        full = [device.to_device(workloads.random_workload(seed + 1000 * r + k, B, Hq, Hkv, D, [c] * B, [N] * B,
                                                           max_depth=13, name="cost")) for k in range(copies)]
        for n in n_values:
            cases = []
            for dw in full:
                w = dw.w
                idx = np.concatenate([np.arange(w.cu_T[b], w.cu_T[b] + n) for b in range(B)])
                sub = dataclasses.replace(w, T=np.full(B, n, np.int64), cu_T=(np.arange(B + 1) * n).astype(np.int32),
                                          parent=np.ascontiguousarray(w.parent[idx]))
                ti = torch.from_numpy(idx).to(dw.q.device)
                d = device.DeviceWorkload(w=sub, q=dw.q[ti].contiguous(), k_tree=dw.k_tree[ti].contiguous(),
                                          v_tree=dw.v_tree[ti].contiguous(), k_cache=dw.k_cache, v_cache=dw.v_cache,
                                          cu_T=torch.from_numpy(sub.cu_T).to(dw.q.device), L=dw.L,
                                          parent=torch.from_numpy(np.ascontiguousarray(sub.parent)).to(dw.q.device),
                                          cu_L=dw.cu_L, page_table=None)
                mask = device.build_mask(d)
                out = torch.empty(d.q.shape, dtype=torch.float32, device=d.q.device)
                lse = torch.empty(d.q.shape[:2], dtype=torch.float32, device=d.q.device)
                args = binding.make_args(q=d.q, k_tree=d.k_tree, v_tree=d.v_tree, k_cache=d.k_cache, v_cache=d.v_cache,
                                         anc_mask=mask, cu_T=d.cu_T, L=d.L, max_T=n, max_L=c, scale=w.scale,
                                         cu_L=d.cu_L, out=out, lse=lse)
                need = binding.workspace_bytes(args)
                ws = torch.empty(max(1, (need + 3) // 4), dtype=torch.float32, device=d.q.device)
                args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel() * 4
                cases.append((args, (d, mask, out, lse, ws)))
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                for args, _ in cases:                      # warm-up, eager
                    binding.tree_verify_attn_raw(args, stream=stream)
                stream.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for args, _ in cases:
                        binding.tree_verify_attn_raw(args, stream=stream)
                for _ in range(3):                         # untimed: clocks and code caches settle
                    g.replay()
                stream.synchronize()
                times = []
                for _ in range(replays):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    flush.fill_(1)
                    e0.record(stream)
                    g.replay()
                    e1.record(stream)
                    e1.synchronize()
                    times.append(e0.elapsed_time(e1) * 1e3 / len(cases))
            # the median: where the same launch runs at two speeds from replay to replay (which CUs the workgroups of
            # a launch smaller than the chip land on), the fastest of a few replays is the less repeatable figure
            table[r - 1, n - 1] = float(np.median(times))
        have = np.array(n_values) - 1
        table[r - 1] = np.interp(np.arange(N), have, table[r - 1, have])
        if log:
            log(f"c={c}: n=1 {table[r-1,0]:.2f} us, n={N} {table[r-1,N-1]:.2f} us")
    return table


def write_table(path: str, table: np.ndarray, B: int, L: int, header_lines=()) -> None:
    M, N = table.shape
    with open(path, "w") as f:
        for h in header_lines:
            f.write("# " + h + "\n")
        f.write(f"# rows: context c = k*{L}, k = 1..{M}; columns: n = 1..{N} tree tokens; microseconds; B = {B}\n")
        for r in range(M):
            f.write(" ".join(f"{x:.3f}" for x in table[r]) + "\n")


def read_table(path: str) -> np.ndarray:
    return np.loadtxt(path, comments="#", ndmin=2)


def make_strictly_increasing(table: np.ndarray, eps: float = 1e-3, max_raise: float = 0.05) -> np.ndarray:
    """Conditions a measured table for Algorithm 1, which needs costs strictly increasing in n: every
    entry is raised to at least its left neighbour plus eps microseconds.  Small dips are real: a tree
    that opens one more row block of workgroups, or crosses to a plan with fewer KV splits, can run up to
    about 3 % faster than the slightly smaller tree before it (the planner's model of a launch is only that
    accurate).  A dip deeper than max_raise (relative) is refused: that would be a launch plan gone wrong,
    which the selection would read as a property of the machine.  Measurement plumbing, not part of the
    method."""
    t = np.array(table, dtype=np.float64, copy=True)
    for k in range(1, t.shape[1]):
        floor = t[:, k - 1] + eps
        worst = float(np.max((floor - t[:, k]) / t[:, k]))
        if worst > max_raise:
            r = int(np.argmax((floor - t[:, k]) / t[:, k]))
            raise ValueError(f"cost table row {r} dips by {100 * worst:.1f} % from n = {k} to n = {k + 1}: "
                             f"{t[r, k - 1]:.3f} -> {t[r, k]:.3f}")
        t[:, k] = np.maximum(t[:, k], floor)
    return t


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n")[0])
    ap.add_argument("--B", type=int, default=1)
    ap.add_argument("--L", type=int, default=256, help="context grid step")
    ap.add_argument("--M", type=int, default=8, help="context grid rows")
    ap.add_argument("--N", type=int, default=72, help="largest number of tree tokens")
    ap.add_argument("--stride", type=int, default=1, help="measure every stride-th n, interpolate between")
    ap.add_argument("--replays", type=int, default=7, help="timed graph replays per grid point (the median is kept)")
    ap.add_argument("--out", required=True)
    a = ap.parse_args(argv)
    t0 = time.time()
    n_values = list(range(1, a.N + 1, a.stride))
    table = measure(a.B, a.L, a.M, a.N, replays=a.replays, n_values=n_values, log=lambda s: print(s, flush=True))
    cmd = "python -m paper_2510_26577_amd.cost_table " + " ".join(sys.argv[1:] if argv is None else argv)
    write_table(a.out, table, a.B, a.L, header_lines=[
        "attention slice of the target cost table S_T(B): tva_tree_verify_attn (split-KV attention + merge), MI355X",
        f"head shape Hq=32 Hkv=8 D=128, bf16, dense cache; median of {a.replays} HIP-graph replays over 8 input copies, caches flushed before each",
        "command: " + cmd])
    print(f"wrote {a.out} in {time.time() - t0:.0f} s", flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
