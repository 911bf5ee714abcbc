"""Thin ctypes binding of the draft-tree construction kernels (include/tva_draft.h): argument marshalling only.
The kernels live in libtva.so (csrc/draft.hip)."""
from __future__ import annotations

import ctypes

from . import binding
from .binding import _check, _p, _stream_ptr

MAX_K, MAX_CANDIDATES, MAX_SUBTREE_NODES = 16, 1024, 2048


class ExpandArgs(ctypes.Structure):
    """Mirror of `struct tva_expand_args`."""
    _fields_ = [("B", ctypes.c_int32), ("V", ctypes.c_int32), ("K", ctypes.c_int32), ("sum_N", ctypes.c_int32),
                ("max_N", ctypes.c_int32), ("cu_N", ctypes.c_void_p), ("score", ctypes.c_void_p), ("logp", ctypes.c_void_p),
                ("ld_logp", ctypes.c_int64), ("cand_score", ctypes.c_void_p), ("cand_parent", ctypes.c_void_p),
                ("cand_token", ctypes.c_void_p), ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
                ("draft_cost_row", ctypes.c_void_p), ("target_cost_one", ctypes.c_double), ("C1", ctypes.c_double),
                ("count", ctypes.c_void_p), ("u_c_at", ctypes.c_void_p), ("count_err_flag", ctypes.c_void_p)]


def _lib():
    lib = binding.load_library()
    if not getattr(lib, "_draft_ready", False):
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.tva_expand_workspace_bytes.restype = ctypes.c_size_t
        lib.tva_expand_workspace_bytes.argtypes = [ctypes.POINTER(ExpandArgs)]
        lib.tva_expand_layer.restype = ctypes.c_int
        lib.tva_expand_layer.argtypes = [ctypes.POINTER(ExpandArgs), vp]
        lib.tva_sizeof_expand_args.restype = ctypes.c_size_t
        lib.tva_tree_select_subtree.restype = ctypes.c_int
        lib.tva_tree_select_subtree.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        lib.tva_tree_rerank_count.restype = ctypes.c_int
        lib.tva_tree_rerank_count.argtypes = [vp, i32, i32, vp, i32, ctypes.c_double, vp, vp, vp, vp, ctypes.c_size_t, vp]
        lib.tva_layer_breadth_count.restype = ctypes.c_int
        lib.tva_layer_breadth_count.argtypes = [vp, i32, i32, vp, ctypes.c_double, ctypes.c_double, vp, vp, vp, vp]
        lib.tva_rerank_workspace_bytes.restype = ctypes.c_size_t
        lib.tva_rerank_workspace_bytes.argtypes = [i32, i32, i32]
        if lib.tva_sizeof_expand_args() != ctypes.sizeof(ExpandArgs):
            raise RuntimeError("libtva.so is stale: rebuild it")
        lib._draft_ready = True
    return lib


def expand_workspace_bytes(B: int, V: int, K: int, sum_N: int) -> int:
    a = ExpandArgs()
    a.B, a.V, a.K, a.sum_N = B, V, K, sum_N
    n = _lib().tva_expand_workspace_bytes(ctypes.byref(a))
    if n == ctypes.c_size_t(-1).value:
        raise binding.TvaError(-2)
    return n


def make_expand_args(*, cu_N, score, logp, K: int, sum_N: int, max_N: int, cand_score, cand_parent, cand_token,
                     workspace=None, workspace_bytes: int = 0, draft_cost_row=None, target_cost_one: float = 0.0,
                     C1: float = 0.0, count=None, u_c_at=None, count_err_flag=None) -> ExpandArgs:
    """count (device int32 [1]) asks for the breadth decision on the sorted candidates in the same call."""
    a = ExpandArgs()
    a.B, a.V, a.K, a.sum_N, a.max_N = cu_N.numel() - 1, int(logp.shape[1]), int(K), int(sum_N), int(max_N)
    a.cu_N, a.score, a.logp, a.ld_logp = _p(cu_N), _p(score), _p(logp), int(logp.stride(0))
    a.cand_score, a.cand_parent, a.cand_token = _p(cand_score), _p(cand_parent), _p(cand_token)
    a.workspace, a.workspace_bytes = _p(workspace), int(workspace_bytes)
    a.draft_cost_row, a.target_cost_one, a.C1 = _p(draft_cost_row), float(target_cost_one), float(C1)
    a.count, a.u_c_at, a.count_err_flag = _p(count), _p(u_c_at), _p(count_err_flag)
    return a


def expand_layer_raw(args: ExpandArgs, stream=None) -> None:
    _check(_lib().tva_expand_layer(ctypes.byref(args), _stream_ptr(stream)))


def expand_layer(cu_N, score, logp, K: int, max_N: int, stream=None):
    """Device tensors in (cu_N int32 [B+1], score float32 [sum_N], logp float32 [sum_N, V]); returns the candidates
    (cand_score float32, cand_parent int32, cand_token int32), each [sum_N * K], sequence b's at cu_N[b] * K ..."""
    import torch
    sum_N, V = int(logp.shape[0]), int(logp.shape[1])
    dev = logp.device
    cs = torch.empty(sum_N * K, dtype=torch.float32, device=dev)
    cp = torch.empty(sum_N * K, dtype=torch.int32, device=dev)
    ct = torch.empty(sum_N * K, dtype=torch.int32, device=dev)
    need = expand_workspace_bytes(cu_N.numel() - 1, V, K, sum_N)
    ws = torch.empty(max(1, need // 8), dtype=torch.int64, device=dev)
    a = make_expand_args(cu_N=cu_N, score=score, logp=logp, K=K, sum_N=sum_N, max_N=max_N, cand_score=cs, cand_parent=cp,
                         cand_token=ct, workspace=ws, workspace_bytes=need)
    expand_layer_raw(a, stream)
    return cs, cp, ct


def select_subtree(score, parent, cu_M, cu_T, max_M: int, old_index=None, new_parent=None, err_flag=None, stream=None,
                   total_kept: int = None):
    """Device tensors in; returns (old_index, new_parent), each int32 [cu_T[B]] (total_kept, a host copy of cu_T[B],
    sizes them when they are not passed)."""
    import torch
    B = cu_M.numel() - 1
    if old_index is None:
        old_index = torch.empty(max(1, total_kept), dtype=torch.int32, device=score.device)
    if new_parent is None:
        new_parent = torch.empty(max(1, total_kept), dtype=torch.int32, device=score.device)
    _check(_lib().tva_tree_select_subtree(_p(score), _p(parent), _p(cu_M), _p(cu_T), B, int(max_M), _p(old_index),
                                          _p(new_parent), _p(err_flag), _stream_ptr(stream)))
    return old_index, new_parent


def rerank_count(tree_scores, cost_row, m: int, C3: float, count=None, cu_T=None, err_flag=None, stream=None, workspace=None):
    """Device tensors in (tree_scores float32 [B, N_tot], cost_row float64 [>= min(N_tot, m)]); returns the device
    tensors (count int32 [1], cu_T int32 [B + 1] = b * count).  workspace: a device tensor of
    tva_rerank_workspace_bytes(B, N_tot, m) bytes (allocated when not passed)."""
    import torch
    B, N_tot = int(tree_scores.shape[0]), int(tree_scores.shape[1])
    if count is None:
        count = torch.empty(1, dtype=torch.int32, device=tree_scores.device)
    if cu_T is None:
        cu_T = torch.empty(B + 1, dtype=torch.int32, device=tree_scores.device)
    if workspace is None:
        need = _lib().tva_rerank_workspace_bytes(B, N_tot, int(m))
        if need == ctypes.c_size_t(-1).value:
            raise binding.TvaError(-1)
        workspace = torch.empty(max(1, need // 4), dtype=torch.float32, device=tree_scores.device)
    _check(_lib().tva_tree_rerank_count(_p(tree_scores), B, N_tot, _p(cost_row), int(m), float(C3), _p(count), _p(cu_T),
                                        _p(err_flag), _p(workspace), workspace.numel() * workspace.element_size(),
                                        _stream_ptr(stream)))
    return count, cu_T


def breadth_count(cand_score, draft_cost_row, target_cost_one: float, C1: float, count=None, u_c_at=None, err_flag=None,
                  stream=None):
    """Device tensors in (cand_score float32 [B, N] in descending order per sample, draft_cost_row float64 [N]);
    returns the device tensors (count int32 [1], u_c_at float64 [2])."""
    import torch
    B, N = int(cand_score.shape[0]), int(cand_score.shape[1])
    if count is None:
        count = torch.empty(1, dtype=torch.int32, device=cand_score.device)
    if u_c_at is None:
        u_c_at = torch.empty(2, dtype=torch.float64, device=cand_score.device)
    _check(_lib().tva_layer_breadth_count(_p(cand_score), B, N, _p(draft_cost_row), float(target_cost_one), float(C1),
                                          _p(count), _p(u_c_at), _p(err_flag), _stream_ptr(stream)))
    return count, u_c_at


def _bench(argv=None) -> int:
    """Times tva_expand_layer and tva_tree_select_subtree on seeded synthetic layers made on the device (log-softmax of
    normal logits) and prints one JSON line per shape.  Plumbing only; the kernels do the work."""
    import argparse
    import json
    import numpy as np
    import torch

    ap = argparse.ArgumentParser(description="time tva_expand_layer and tva_tree_select_subtree")
    ap.add_argument("--steps", type=int, default=64)
    a = ap.parse_args(argv)
    assert torch.cuda.is_available(), "needs a GPU"
    gen = torch.Generator(device="cuda")
    gen.manual_seed(79)
    stream = torch.cuda.Stream()
    flush = torch.empty(1 << 28, dtype=torch.int32, device="cuda")

    def timed(run, calls):
        with torch.cuda.stream(stream):
            run()
            stream.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=stream):
                for _ in range(max(1, a.steps // calls)):
                    run()
            g.replay()
            stream.synchronize()
            ts = []
            for _ in range(5):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                flush.fill_(1)
                e0.record(stream)
                g.replay()
                e1.record(stream)
                e1.synchronize()
                ts.append(e0.elapsed_time(e1) * 1e3 / (max(1, a.steps // calls) * calls))
        return float(np.median(ts))

    for B, n, V, K in ((1, 12, 32000, 12), (1, 12, 128256, 12), (8, 12, 128256, 12), (64, 12, 32000, 12), (64, 12, 128256, 12),
                       (16, 48, 128256, 8)):
        copies = 4 if B * n * V * 4 < (1 << 29) else 2
        cases = []
        for _ in range(copies):
            logp = torch.log_softmax(torch.randn((B * n, V), generator=gen, device="cuda") * 3.0, dim=1)
            score = -torch.rand(B * n, generator=gen, device="cuda") * 4.0
            cu_N = (torch.arange(B + 1, device="cuda") * n).to(torch.int32)
            need = expand_workspace_bytes(B, V, K, B * n)
            ws = torch.empty(max(1, need // 8), dtype=torch.int64, device="cuda")
            outs = (torch.empty(B * n * K, dtype=torch.float32, device="cuda"), torch.empty(B * n * K, dtype=torch.int32, device="cuda"),
                    torch.empty(B * n * K, dtype=torch.int32, device="cuda"))
            dcost = torch.cumsum(torch.rand(n * K, dtype=torch.float64, device="cuda") * 0.04 + 0.002, 0) + 0.5
            cnt = (torch.zeros(1, dtype=torch.int32, device="cuda"), torch.zeros(2, dtype=torch.float64, device="cuda"))
            common = dict(cu_N=cu_N, score=score, logp=logp, K=K, sum_N=B * n, max_N=n, cand_score=outs[0], cand_parent=outs[1],
                          cand_token=outs[2], workspace=ws, workspace_bytes=need)
            cases.append((make_expand_args(**common),
                          (logp, score, cu_N, ws, outs, dcost, cnt),
                          make_expand_args(draft_cost_row=dcost, target_cost_one=8.0, C1=0.01, count=cnt[0], u_c_at=cnt[1], **common)))
        us = timed(lambda: [expand_layer_raw(c[0], stream) for c in cases], copies)
        us_counted = timed(lambda: [expand_layer_raw(c[2], stream) for c in cases], copies) if n * K <= 1024 else None
        nbytes = 4.0 * B * n * V
        print(json.dumps({"kernel": "tva_expand_layer", "shape": f"B={B} rows/seq={n} V={V} K={K}", "us_per_call": us,
                          "us_with_the_breadth_decision": us_counted,
                          "logp_bytes": nbytes, "GBps": nbytes / (us * 1e-6) / 1e9, "frac_of_8TBps": nbytes / (us * 1e-6) / 8e12}),
              flush=True)
        del cases
        torch.cuda.empty_cache()

    for B in (1, 8, 64):
        N = 144
        cand = -torch.sort(-torch.exp(-torch.rand((B, N), generator=gen, device="cuda") * 6.0), dim=1).values.contiguous()
        dcost = torch.cumsum(torch.rand(N, dtype=torch.float64, device="cuda") * 0.04 + 0.002, 0) + 0.5
        count = torch.zeros(1, dtype=torch.int32, device="cuda")
        at = torch.zeros(2, dtype=torch.float64, device="cuda")
        us = timed(lambda: breadth_count(cand, dcost, 8.0, 1.0, count=count, u_c_at=at, stream=stream), 1)
        print(json.dumps({"kernel": "tva_layer_breadth_count", "shape": f"B={B} candidates={N}", "us_per_call": us,
                          "count": int(count.item())}), flush=True)

    rng = np.random.Generator(np.random.PCG64(80))
    for B, M, keep in ((1, 145, 60), (8, 145, 60), (64, 145, 32), (8, 1024, 72)):
        parent = np.concatenate([np.array([-1] + [int(rng.integers(max(0, i - 9), i)) for i in range(1, M)], np.int32) for _ in range(B)])
        score = np.zeros(B * M, np.float32)
        for b in range(B):
            for i in range(1, M):
                score[b * M + i] = score[b * M + parent[b * M + i]] - np.float32(rng.exponential(0.7))
        d = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
        ds, dp = d(score), d(parent)
        cu_M = (torch.arange(B + 1, device="cuda") * M).to(torch.int32)
        cu_T = (torch.arange(B + 1, device="cuda") * keep).to(torch.int32)
        old = torch.empty(B * keep, dtype=torch.int32, device="cuda")
        newp = torch.empty(B * keep, dtype=torch.int32, device="cuda")
        us = timed(lambda: select_subtree(ds, dp, cu_M, cu_T, M, old_index=old, new_parent=newp, stream=stream), 1)
        print(json.dumps({"kernel": "tva_tree_select_subtree", "shape": f"B={B} nodes={M} keep={keep}", "us_per_call": us}), flush=True)
        if True:
            # the count of nodes to keep, then the cut with the prefix array it wrote (room for the most it may keep)
            cost = torch.cumsum(torch.rand(72, dtype=torch.float64, device="cuda") * 0.05 + 0.01, 0) + 5.0
            count = torch.zeros(1, dtype=torch.int32, device="cuda")
            cu_K = torch.zeros(B + 1, dtype=torch.int32, device="cuda")
            old2 = torch.empty(B * 72, dtype=torch.int32, device="cuda")
            newp2 = torch.empty(B * 72, dtype=torch.int32, device="cuda")
            scores2 = (-ds).reshape(B, M)
            rws = torch.empty(B * 72, dtype=torch.float32, device="cuda")
            us = timed(lambda: rerank_count(scores2, cost, 72, 30.0, count=count, cu_T=cu_K, stream=stream, workspace=rws), 1)
            kept = int(count.item())

            def both():
                rerank_count(scores2, cost, 72, 30.0, count=count, cu_T=cu_K, stream=stream, workspace=rws)
                select_subtree(ds, dp, cu_M, cu_K, M, old_index=old2, new_parent=newp2, stream=stream)
            us2 = timed(both, 1)
            print(json.dumps({"kernel": "tva_tree_rerank_count", "shape": f"B={B} nodes={M} m=72", "us_per_call": us, "count": kept,
                              "us_with_the_cut_behind_it": us2}), flush=True)
    return 0


if __name__ == "__main__":
    import sys
    sys.exit(_bench())
