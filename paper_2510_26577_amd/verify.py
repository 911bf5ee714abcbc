"""Thin ctypes binding of include/tva_verify.h (argument marshalling only): greedy acceptance of a
root path per draft tree and commit of the accepted nodes' K/V rows to the cache.  Both run as HIP
kernels in libtva.so; a missing library raises (no fallback)."""
from __future__ import annotations

import ctypes

from . import binding
from .binding import _check, _p, _stream_ptr

_ready = False


class CommitArgs(ctypes.Structure):
    """Mirror of `struct tva_commit_args`."""
    _fields_ = [
        ("B", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32), ("max_path", ctypes.c_int32),
        ("cu_T", ctypes.c_void_p), ("L", ctypes.c_void_p), ("path", ctypes.c_void_p), ("path_len", ctypes.c_void_p),
        ("k_tree", ctypes.c_void_p), ("v_tree", ctypes.c_void_p), ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
        ("cu_L", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("stride_page", ctypes.c_int64), ("stride_tok", ctypes.c_int64), ("stride_head", ctypes.c_int64),
        ("L_out", ctypes.c_void_p), ("err_flag", ctypes.c_void_p),
        ("n_layers", ctypes.c_int32), ("layer_stride_cache", ctypes.c_int64), ("layer_stride_tree", ctypes.c_int64),
    ]


class SampleArgs(ctypes.Structure):
    """Mirror of `struct tva_sample_args`."""
    _fields_ = [("B", ctypes.c_int32), ("V", ctypes.c_int32), ("max_path", ctypes.c_int32)] + \
               [(n, ctypes.c_void_p) for n in ("parent", "cu_T", "draft_token", "p_target", "q_draft", "u", "u_final",
                                               "residual", "path", "path_len", "next_token", "err_flag", "workspace")] + \
               [("workspace_bytes", ctypes.c_size_t), ("workgroups_per_sequence", ctypes.c_int32), ("sum_T", ctypes.c_int32),
                ("unit_rows", ctypes.c_int32)]


def _lib():
    global _ready
    lib = binding.load_library()
    if not _ready:
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.tva_accept_greedy.restype = ctypes.c_int
        lib.tva_accept_greedy.argtypes = [vp, vp, vp, vp, i32, i32, vp, vp, vp, vp]
        lib.tva_commit_path.restype = ctypes.c_int
        lib.tva_commit_path.argtypes = [ctypes.POINTER(CommitArgs), vp]
        lib.tva_sizeof_commit_args.restype = ctypes.c_size_t
        lib.tva_accept_sampling.restype = ctypes.c_int
        lib.tva_accept_sampling.argtypes = [ctypes.POINTER(SampleArgs), vp]
        lib.tva_sizeof_sample_args.restype = ctypes.c_size_t
        lib.tva_accept_sampling_wait_bound_test.restype = ctypes.c_int
        lib.tva_accept_sampling_wait_bound_test.argtypes = [ctypes.POINTER(SampleArgs), ctypes.c_int32, vp]
        lib.tva_sample_workspace_bytes.restype = ctypes.c_size_t
        lib.tva_sample_workspace_bytes.argtypes = [ctypes.c_int32]
        lib.tva_sample_workspace_bytes_rows.restype = ctypes.c_size_t
        lib.tva_sample_workspace_bytes_rows.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
        if lib.tva_sizeof_sample_args() != ctypes.sizeof(SampleArgs):
            raise RuntimeError("libtva.so is stale: rebuild it")
        if lib.tva_sizeof_commit_args() != ctypes.sizeof(CommitArgs):
            raise RuntimeError("libtva.so is stale: rebuild it")
        _ready = True
    return lib


def accept_greedy(parent, cu_T, draft_token, target_token, max_path: int, path=None, path_len=None, next_token=None,
                  stream=None):
    """Device int32 tensors in; returns (path [B, max_path], path_len [B], next_token [B])."""
    import torch
    B = cu_T.numel() - 1
    dev = cu_T.device
    if path is None:
        path = torch.full((B, max_path), -1, dtype=torch.int32, device=dev)
    if path_len is None:
        path_len = torch.empty(B, dtype=torch.int32, device=dev)
    if next_token is None:
        next_token = torch.empty(B, dtype=torch.int32, device=dev)
    _check(_lib().tva_accept_greedy(_p(parent), _p(cu_T), _p(draft_token), _p(target_token), B, int(max_path),
                                    _p(path), _p(path_len), _p(next_token), _stream_ptr(stream)))
    return path, path_len, next_token


def accept_sampling(parent, cu_T, draft_token, p_target, q_draft, u, u_final, max_path: int, residual=None,
                    err_flag=None, stream=None, workspace="auto", workgroups_per_sequence: int = 0, wait_bound_test_spins: int = 0,
                    sum_T: int = 0, unit_rows: bool = False):
    """Device tensors in (int32 trees and tokens, float32 distributions [sum_T, V] and uniform numbers); returns
    (path [B, max_path], path_len [B], next_token [B]).  workspace: "auto" allocates the one that lets several
    workgroups share a sequence (and, with sum_T, holds the row sums made ahead of the walk), None runs one
    workgroup per sequence, or a device tensor of tva_sample_workspace_bytes[_rows] bytes.  sum_T: the host's
    count of the batch's nodes (cu_T[B]), or 0."""
    import torch
    B, V = cu_T.numel() - 1, int(p_target.shape[1])
    dev = cu_T.device
    path = torch.full((B, max_path), -1, dtype=torch.int32, device=dev)
    path_len = torch.empty(B, dtype=torch.int32, device=dev)
    next_token = torch.empty(B, dtype=torch.int32, device=dev)
    if residual is None:
        residual = torch.empty((max(B, 1), V), dtype=torch.float32, device=dev)
    a = SampleArgs()
    a.B, a.V, a.max_path = B, V, int(max_path)
    a.parent, a.cu_T, a.draft_token = _p(parent), _p(cu_T), _p(draft_token)
    a.p_target, a.q_draft, a.u, a.u_final = _p(p_target), _p(q_draft), _p(u), _p(u_final)
    a.residual, a.path, a.path_len, a.next_token, a.err_flag = _p(residual), _p(path), _p(path_len), _p(next_token), _p(err_flag)
    if isinstance(workspace, str):
        workspace = torch.empty(max(1, _lib().tva_sample_workspace_bytes_rows(B, int(sum_T), V) // 8), dtype=torch.int64,
                                device=dev)
    if workspace is not None:
        a.workspace, a.workspace_bytes = _p(workspace), workspace.numel() * workspace.element_size()
    a.workgroups_per_sequence = int(workgroups_per_sequence)
    a.sum_T = int(sum_T)
    a.unit_rows = int(bool(unit_rows))
    if wait_bound_test_spins:                 # (tests of the bounded wait: every wait misses one arrival and gives up)
        _check(_lib().tva_accept_sampling_wait_bound_test(ctypes.byref(a), int(wait_bound_test_spins), _stream_ptr(stream)))
    else:
        _check(_lib().tva_accept_sampling(ctypes.byref(a), _stream_ptr(stream)))
    return path, path_len, next_token


def make_commit_args(*, cu_T, L, path, path_len, k_tree, v_tree, k_cache, v_cache, cu_L=None, page_table=None,
                     page_size: int = 0, strides=(0, 0, 0), L_out=None, err_flag=None, n_layers: int = 0,
                     layer_stride_cache: int = 0, layer_stride_tree: int = 0) -> CommitArgs:
    """k_cache, v_cache (and k_tree, v_tree): one layer's tensors, or with n_layers > 1 the first layer's, the others
    layer_stride_* elements further on each."""
    a = CommitArgs()
    a.B = cu_T.numel() - 1
    a.Hkv, a.D = int(k_cache.shape[-2]), int(k_cache.shape[-1])
    a.max_path = int(path.shape[1])
    a.cu_T, a.L, a.path, a.path_len = _p(cu_T), _p(L), _p(path), _p(path_len)
    a.k_tree, a.v_tree, a.k_cache, a.v_cache = _p(k_tree), _p(v_tree), _p(k_cache), _p(v_cache)
    a.cu_L, a.page_table = _p(cu_L), _p(page_table)
    a.page_size = int(page_size)
    a.max_pages = int(page_table.shape[1]) if page_table is not None else 0
    a.stride_page, a.stride_tok, a.stride_head = (int(s) for s in strides)
    if k_cache.element_size() == 1:
        # 8-bit K/V: the kernels only move bytes, so a row of D bytes is passed as D/2 two-byte elements
        assert a.D % 2 == 0 and all(int(s) % 2 == 0 for s in strides)
        a.D //= 2
        a.stride_page, a.stride_tok, a.stride_head = (int(s) // 2 for s in strides)
        assert layer_stride_cache % 2 == 0 and layer_stride_tree % 2 == 0
        layer_stride_cache, layer_stride_tree = layer_stride_cache // 2, layer_stride_tree // 2
    a.n_layers, a.layer_stride_cache, a.layer_stride_tree = int(n_layers), int(layer_stride_cache), int(layer_stride_tree)
    a.L_out, a.err_flag = _p(L_out), _p(err_flag)
    # the struct holds raw addresses: keep the tensors alive as long as it lives
    a._keep = (cu_T, L, path, path_len, k_tree, v_tree, k_cache, v_cache, cu_L, page_table, L_out, err_flag)
    return a


def commit_path_raw(args: CommitArgs, stream=None) -> None:
    _check(_lib().tva_commit_path(ctypes.byref(args), _stream_ptr(stream)))


def commit_path(**kw):
    """Keyword arguments of make_commit_args plus stream; writes the caches in place."""
    stream = kw.pop("stream", None)
    commit_path_raw(make_commit_args(**kw), stream)


def _bench(argv=None) -> int:
    """Times the two kernels on seeded synthetic steps of the benchmark's shapes (HIP-graph replay over
    rotating copies) and prints one JSON line per shape.  Plumbing only; the kernels do the work."""
    import argparse
    import json
    import numpy as np
    import torch
    from . import workloads as wl

    ap = argparse.ArgumentParser(description="time tva_accept_greedy and tva_commit_path")
    ap.add_argument("--steps", type=int, default=64)
    a = ap.parse_args(argv)
    assert torch.cuda.is_available(), "needs a GPU"
    rng = np.random.Generator(np.random.PCG64(77))
    stream = torch.cuda.Stream()
    for name, B, T, Hkv, D, depth in (("B=1 T=60", 1, 60, 8, 128, 6), ("B=8 T=32", 8, 32, 8, 128, 6),
                                      ("B=64 T=8", 64, 8, 8, 128, 8), ("B=64 T=72", 64, 72, 8, 128, 13)):
        copies = 8
        cases = []
        accepted = 0
        for c in range(copies):
            trees = [wl.tree_uniform(rng, T, depth) for _ in range(B)]
            parent = np.concatenate(trees).astype(np.int32)
            cu_T = (np.arange(B + 1) * T).astype(np.int32)
            draft = rng.integers(0, 1 << 15, B * T).astype(np.int32)
            target = rng.integers(0, 1 << 15, B * T).astype(np.int32)
            for b in range(B):                       # plant a matching child under most nodes: long accepted paths
                for i in range(T):
                    kids = np.nonzero(trees[b] == i)[0]
                    if len(kids) and rng.random() < 0.85:
                        target[b * T + i] = draft[b * T + int(kids[0])]
            L = np.full(B, 1024, np.int32)
            cap = L + T
            cu_L = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
            d = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
            kt = torch.randint(-30000, 30000, (B * T, Hkv, D), dtype=torch.int16, device="cuda")
            vt = torch.randint(-30000, 30000, (B * T, Hkv, D), dtype=torch.int16, device="cuda")
            kc = torch.zeros((int(cap.sum()), Hkv, D), dtype=torch.int16, device="cuda")
            vc = torch.zeros_like(kc)
            path = torch.full((B, depth + 1), -1, dtype=torch.int32, device="cuda")
            plen = torch.zeros(B, dtype=torch.int32, device="cuda")
            nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
            acc = (d(parent), d(cu_T), d(draft), d(target), path, plen, nxt)
            cargs = make_commit_args(cu_T=acc[1], L=d(L), path=path, path_len=plen, k_tree=kt, v_tree=vt, k_cache=kc,
                                     v_cache=vc, cu_L=d(cu_L))
            cases.append((acc, cargs, (kt, vt, kc, vc)))

        def run(which):
            for acc, cargs, _ in cases:
                if which in ("accept", "both"):
                    accept_greedy(acc[0], acc[1], acc[2], acc[3], depth + 1, path=acc[4], path_len=acc[5],
                                  next_token=acc[6], stream=stream)
                if which in ("commit", "both"):
                    commit_path_raw(cargs, stream)

        times = {}
        with torch.cuda.stream(stream):
            run("both")
            stream.synchronize()
            accepted = sum(int(c[0][5].sum().item()) for c in cases) / copies
            for which in ("accept", "commit", "both"):
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for _ in range(a.steps // copies):
                        run(which)
                g.replay()
                stream.synchronize()
                best = 1e30
                for _ in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    g.replay()
                    e1.record(stream)
                    e1.synchronize()
                    best = min(best, e0.elapsed_time(e1) * 1e3 / (a.steps // copies * copies))
                times[which] = best
        moved = accepted * Hkv * D * 2 * 2 * 2      # K and V rows, read + write
        print(json.dumps({"shape": name, "accepted_nodes_per_step": accepted, "accept_us": times["accept"],
                          "commit_us": times["commit"], "both_us": times["both"], "commit_bytes": moved,
                          "commit_GBps": moved / (times["commit"] * 1e-6) / 1e9}), flush=True)
    _bench_layers(a.steps)
    _bench_sampling(a.steps)
    return 0


def _bench_layers(steps: int) -> None:
    """The commit of a whole model's layers: 32 calls of tva_commit_path against one call with n_layers = 32 (the
    caches of the layers one allocation, a layer's tensors a fixed stride apart)."""
    import json
    import numpy as np
    import torch
    from . import workloads as wl

    rng = np.random.Generator(np.random.PCG64(81))
    stream = torch.cuda.Stream()
    layers, Hkv, D = 32, 8, 128
    for name, B, T, depth in (("B=1 T=60", 1, 60, 6), ("B=8 T=32", 8, 32, 6), ("B=64 T=8", 64, 8, 8)):
        trees = [wl.tree_uniform(rng, T, depth) for _ in range(B)]
        parent = np.concatenate(trees).astype(np.int32)
        cu_T = (np.arange(B + 1) * T).astype(np.int32)
        path = np.full((B, depth + 1), -1, np.int32)
        plen = np.zeros(B, np.int32)
        for b in range(B):                          # a root path: from a random leaf upwards
            node, up = int(rng.integers(0, T)), []
            while node >= 0:
                up.append(node)
                node = int(trees[b][node])
            up = up[::-1][:depth + 1]
            path[b, :len(up)], plen[b] = up, len(up)
        L = np.full(B, 1024, np.int32)
        cu_L = (np.arange(B + 1) * (1024 + T)).astype(np.int32)
        d = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
        rows = B * (1024 + T)
        kc = torch.zeros((layers, rows, Hkv, D), dtype=torch.int16, device="cuda")
        vc = torch.zeros_like(kc)
        kt = torch.randint(-30000, 30000, (layers, B * T, Hkv, D), dtype=torch.int16, device="cuda")
        vt = torch.randint(-30000, 30000, (layers, B * T, Hkv, D), dtype=torch.int16, device="cuda")
        common = dict(cu_T=d(cu_T), L=d(L), path=d(path), path_len=d(plen), cu_L=d(cu_L))
        each = [make_commit_args(k_tree=kt[l], v_tree=vt[l], k_cache=kc[l], v_cache=vc[l], **common) for l in range(layers)]
        one = make_commit_args(k_tree=kt[0], v_tree=vt[0], k_cache=kc[0], v_cache=vc[0], n_layers=layers,
                               layer_stride_cache=rows * Hkv * D, layer_stride_tree=B * T * Hkv * D, **common)
        times = {}
        for form, run in (("calls", lambda: [commit_path_raw(c, stream) for c in each]), ("one", lambda: commit_path_raw(one, stream))):
            with torch.cuda.stream(stream):
                run()
                stream.synchronize()
                g = torch.cuda.CUDAGraph()
                reps = max(1, steps // 8)
                with torch.cuda.graph(g, stream=stream):
                    for _ in range(reps):
                        run()
                g.replay()
                stream.synchronize()
                best = 1e30
                for _ in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    g.replay()
                    e1.record(stream)
                    e1.synchronize()
                    best = min(best, e0.elapsed_time(e1) * 1e3 / reps)
            times[form] = best
        moved = float(plen.sum()) * layers * Hkv * D * 2 * 2 * 2
        print(json.dumps({"shape": name + f" layers={layers}", "accepted_nodes": int(plen.sum()), "commit_us_one_call_per_layer": times["calls"],
                          "commit_us_one_call": times["one"], "commit_bytes": moved,
                          "commit_GBps_one_call": moved / (times["one"] * 1e-6) / 1e9}), flush=True)


def _bench_sampling(steps: int) -> None:
    """Times tva_accept_sampling on seeded synthetic steps made on the device (softmax of normal logits, the draft's
    logits the target's plus noise, tokens drawn from the parent's draft row) and prints one JSON line per shape with
    the vocabulary passes the walks took (counted on the host from the returned paths and the trees)."""
    import json
    import numpy as np
    import torch
    from . import workloads as wl

    rng = np.random.Generator(np.random.PCG64(78))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(78)
    stream = torch.cuda.Stream()
    for name, B, T, V, depth in (("B=1 T=60 V=32000", 1, 60, 32000, 6), ("B=1 T=60 V=128256", 1, 60, 128256, 6),
                                 ("B=1 T=8 V=128256", 1, 8, 128256, 6), ("B=4 T=16 V=128256", 4, 16, 128256, 6),
                                 ("B=8 T=8 V=128256", 8, 8, 128256, 6),
                                 ("B=8 T=32 V=128256", 8, 32, 128256, 6), ("B=64 T=8 V=128256", 64, 8, 128256, 8),
                                 ("B=64 T=60 V=32000", 64, 60, 32000, 6)):
        copies = 4
        cases, sums, rejs = [], 0, 0
        for c in range(copies):
            trees = [wl.tree_expand_prune(rng, T, depth=depth) for _ in range(B)]
            parent = np.concatenate(trees).astype(np.int32)
            cu_T = (np.arange(B + 1) * T).astype(np.int32)
            logit = torch.randn((B * T, V), generator=gen, device="cuda") * 3.0
            p = torch.softmax(logit, dim=1)
            q = torch.softmax(logit + 0.5 * torch.randn((B * T, V), generator=gen, device="cuda"), dim=1)
            del logit
            up = torch.from_numpy(np.concatenate([np.maximum(t, 0) + b * T for b, t in enumerate(trees)])).cuda()
            tok = torch.multinomial(q[up], 1, generator=gen).reshape(-1).to(torch.int32)
            d = lambda x: torch.from_numpy(np.ascontiguousarray(x)).cuda()
            case = dict(parent=d(parent), cu_T=d(cu_T), tok=tok, p=p, q=q,
                        u=torch.rand(B * T, generator=gen, device="cuda"), uf=torch.rand(B, generator=gen, device="cuda"),
                        residual=torch.empty((B, V), dtype=torch.float32, device="cuda"),
                        flag=torch.zeros(1, dtype=torch.int32, device="cuda"),
                        ws=torch.empty(max(1, _lib().tva_sample_workspace_bytes_rows(B, B * T, V) // 8), dtype=torch.int64,
                                       device="cuda"))
            path, plen, _ = accept_sampling(case["parent"], case["cu_T"], tok, p, q, case["u"], case["uf"], depth + 1,
                                            residual=case["residual"], err_flag=case["flag"], workspace=case["ws"])
            torch.cuda.synchronize()
            assert int(case["flag"].item()) == 0
            path, plen = path.cpu().numpy(), plen.cpu().numpy()
            for b in range(B):                      # one sum per accepted node; one residual per child refused under it
                for j in range(int(plen[b])):
                    sums += 1
                    kids = np.nonzero(trees[b] == path[b, j])[0]
                    if j + 1 < int(plen[b]):
                        rejs += int((kids < path[b, j + 1]).sum())
                    elif int(plen[b]) < depth + 1:
                        rejs += len(kids)
            cases.append(case)
        sums, rejs = sums / copies, rejs / copies

        # the three forms: row sums ahead of the walk where the library sees fit (the host's node count given), several
        # workgroups per sequence without them, one workgroup per sequence
        def run(form):
            for k in cases:
                accept_sampling(k["parent"], k["cu_T"], k["tok"], k["p"], k["q"], k["u"], k["uf"], depth + 1,
                                residual=k["residual"], err_flag=k["flag"], stream=stream,
                                workspace=None if form == "one" else k["ws"], sum_T=B * T if form in ("ahead", "unit") else 0,
                                unit_rows=form == "unit")

        times = {}
        for shared in ("unit", "ahead", "shared", "one"):
            with torch.cuda.stream(stream):
                run(shared)
                stream.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    for _ in range(max(1, steps // copies)):
                        run(shared)
                g.replay()
                stream.synchronize()
                best = 1e30
                for _ in range(5):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    g.replay()
                    e1.record(stream)
                    e1.synchronize()
                    best = min(best, e0.elapsed_time(e1) * 1e3 / (max(1, steps // copies) * copies))
            times[shared] = best
            assert all(int(k["flag"].item()) == 0 for k in cases)
        moved = 4.0 * V * (sums + 3 * rejs + B / 16.0)   # a sum reads a row; a residual reads two and writes one; the draw a segment
        print(json.dumps({"shape": name, "accepted_nodes_per_step": sums, "refused_children_per_step": rejs,
                          "sampling_us": times["ahead"], "sampling_us_rows_taken_as_distributions": times["unit"],
                          "sampling_us_without_the_node_count": times["shared"],
                          "sampling_us_one_workgroup_per_sequence": times["one"],
                          "vocabulary_bytes": moved, "GBps": moved / (times["shared"] * 1e-6) / 1e9}), flush=True)
        del cases
        torch.cuda.empty_cache()


if __name__ == "__main__":
    import sys
    sys.exit(_bench())
