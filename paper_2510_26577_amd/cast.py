"""Thin ctypes binding of the host entry points of include/tva_cast.h (argument marshalling only:
numpy arrays -> host pointers).  The selection logic itself runs in libtva.so (csrc/cast.cpp);
if the library is missing, loading raises -- there is no Python fallback."""
from __future__ import annotations

import ctypes

import numpy as np

from . import binding

_ready = False


def _lib():
    global _ready
    lib = binding.load_library()
    if not _ready:
        i32, f64, vp = ctypes.c_int32, ctypes.c_double, ctypes.c_void_p
        lib.tva_cast_select_context.restype = i32
        lib.tva_cast_select_context.argtypes = [i32, i32, i32]
        lib.tva_cast_select_max_valid_index.restype = i32
        lib.tva_cast_select_max_valid_index.argtypes = [vp, vp, i32, f64]
        lib.tva_cast_layer_utility.restype = ctypes.c_int
        lib.tva_cast_layer_utility.argtypes = [vp, i32, i32, vp]
        lib.tva_cast_layer_cost.restype = ctypes.c_int
        lib.tva_cast_layer_cost.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp]
        lib.tva_cast_breadth_prune.restype = i32
        lib.tva_cast_breadth_prune.argtypes = [vp, i32, i32, vp, vp, i32, i32, i32, i32, f64, vp, vp, vp]
        lib.tva_cast_depth_bytes.restype = ctypes.c_size_t
        lib.tva_cast_depth_bytes.argtypes = [i32, i32]
        lib.tva_cast_depth_init.restype = ctypes.c_int
        lib.tva_cast_depth_init.argtypes = [vp, i32, i32, f64]
        lib.tva_cast_depth_alpha.restype = f64
        lib.tva_cast_depth_alpha.argtypes = [vp, i32]
        lib.tva_cast_depth_should_expand.restype = ctypes.c_int
        lib.tva_cast_depth_should_expand.argtypes = [vp, i32, f64, f64]
        lib.tva_cast_depth_update.restype = f64
        lib.tva_cast_depth_update.argtypes = [vp, i32, f64, f64]
        lib.tva_cast_expansion_plan.restype = i32
        lib.tva_cast_expansion_plan.argtypes = [vp, vp, i32, i32, vp, vp, i32, i32, i32, i32, f64, vp, vp, vp]
        lib.tva_cast_rerank_count.restype = i32
        lib.tva_cast_rerank_count.argtypes = [vp, i32, i32, vp, i32, i32, i32, i32, i32, f64, vp]
        lib.tva_cast_select_subtree.restype = ctypes.c_int
        lib.tva_cast_select_subtree.argtypes = [vp, vp, i32, i32, vp, vp, vp]
        _ready = True
    return lib


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _count(code: int) -> int:
    if code < 1:
        raise binding.TvaError(code)
    return code


def _table(S):
    S = _f64(S)
    assert S.ndim == 2
    return S


def select_context(c: int, L: int, M: int) -> int:
    return _count(_lib().tva_cast_select_context(c, L, M))


def select_max_valid_index(u, c, C: float) -> int:
    u, c = _f64(u), _f64(c)
    assert u.shape == c.shape and u.ndim == 1
    return _count(_lib().tva_cast_select_max_valid_index(_p(u), _p(c), len(u), C))


def layer_utility(scores) -> np.ndarray:
    s = _f32(scores)
    u = np.empty(s.shape[1], np.float64)
    binding._check(_lib().tva_cast_layer_utility(_p(s), s.shape[0], s.shape[1], _p(u)))
    return u


def layer_cost(S_D, S_T, ctx: int, L: int, n_candidates: int) -> np.ndarray:
    S_D, S_T = _table(S_D), _table(S_T)
    c = np.empty(n_candidates, np.float64)
    binding._check(_lib().tva_cast_layer_cost(_p(S_D), _p(S_T), S_D.shape[0], S_D.shape[1], L, ctx, n_candidates, _p(c)))
    return c


def breadth_prune(scores, S_D, S_T, ctx: int, L: int, C1: float):
    s, S_D, S_T = _f32(scores), _table(S_D), _table(S_T)
    u_at, c_at = ctypes.c_double(), ctypes.c_double()
    work = np.empty(2 * s.shape[1], np.float64)
    n_i = _count(_lib().tva_cast_breadth_prune(_p(s), s.shape[0], s.shape[1], _p(S_D), _p(S_T), S_D.shape[0],
                                               S_D.shape[1], L, ctx, C1, ctypes.byref(u_at), ctypes.byref(c_at), _p(work)))
    return n_i, u_at.value, c_at.value


class DepthPruner:
    """Owns the caller-side state block of the depth-pruning buffers."""

    def __init__(self, max_layers: int, R: int, C2: float):
        n = _lib().tva_cast_depth_bytes(max_layers, R)
        if n == 0:
            raise binding.TvaError(-1)
        self._mem = np.zeros((n + 7) // 8, np.float64)  # 8-byte aligned host memory
        binding._check(_lib().tva_cast_depth_init(_p(self._mem), max_layers, R, C2))

    @property
    def state(self):
        return _p(self._mem)

    def alpha(self, layer: int) -> float:
        return _lib().tva_cast_depth_alpha(self.state, layer)

    def should_expand(self, layer: int, u_ni: float, c_ni: float) -> bool:
        rc = _lib().tva_cast_depth_should_expand(self.state, layer, u_ni, c_ni)
        if rc < 0:
            raise binding.TvaError(rc)
        return bool(rc)

    def update(self, layer: int, u_next: float, u_cur: float) -> float:
        return _lib().tva_cast_depth_update(self.state, layer, u_next, u_cur)


def expansion_plan(layers, S_D, S_T, n0: int, L: int, C1: float, pruner: DepthPruner):
    mats = [_f32(m) for m in layers]
    B = mats[0].shape[0]
    N_i = np.array([m.shape[1] for m in mats], np.int32)
    flat = np.concatenate([m.ravel() for m in mats])
    S_D, S_T = _table(S_D), _table(S_T)
    kept = np.zeros(len(mats), np.int32)
    work = np.empty(2 * int(N_i.max()), np.float64)
    n = _count(_lib().tva_cast_expansion_plan(_p(flat), _p(N_i), len(mats), B, _p(S_D), _p(S_T), S_D.shape[0],
                                              S_D.shape[1], L, n0, C1, pruner.state, _p(kept), _p(work)))
    return [int(x) for x in kept[:n]]


def rerank_count(tree_scores, S_T, n0: int, L: int, m: int, C3: float) -> int:
    s, S_T = _f32(tree_scores), _table(S_T)
    B, N_tot = s.shape
    work = np.empty(B * N_tot + 2 * min(N_tot, m), np.float64)
    return _count(_lib().tva_cast_rerank_count(_p(s), B, N_tot, _p(S_T), S_T.shape[0], S_T.shape[1], L, n0, m, C3, _p(work)))


def select_subtree(score, parent, keep: int):
    s = _f32(score)
    par = np.ascontiguousarray(parent, dtype=np.int32)
    old = np.empty(keep, np.int32)
    newp = np.empty(keep, np.int32)
    work = np.empty(len(s), np.int32)
    binding._check(_lib().tva_cast_select_subtree(_p(s), _p(par), len(s), keep, _p(old), _p(newp), _p(work)))
    return old, newp


def _bench(argv=None) -> int:
    """Times the host entry points at the paper's sizes (K = 12 children of up to 12 nodes per layer, trees grown to
    145 nodes and cut to 72, cost tables of 8 context rows x 160 sizes) on this machine's CPU: one JSON line per
    call, microseconds per call including the ctypes call itself (pointers marshalled once, outside the loop)."""
    import argparse
    import json
    import time

    ap = argparse.ArgumentParser(description="time the host side of the method (no GPU needed)")
    ap.add_argument("--calls", type=int, default=20000)
    a = ap.parse_args(argv)
    lib = _lib()
    rng = np.random.Generator(np.random.PCG64(9))
    M, N_table, L, n0 = 8, 160, 256, 300
    S_T = np.cumsum(rng.uniform(0.02, 0.2, (M, N_table)), axis=1) + 10.0 + np.arange(M)[:, None]
    S_D = np.cumsum(rng.uniform(0.005, 0.05, (M, N_table)), axis=1) + 1.0
    out = []

    def timed(name, call):
        call()
        t0 = time.perf_counter()
        for _ in range(a.calls):
            call()
        us = (time.perf_counter() - t0) / a.calls * 1e6
        out.append({"call": name, "us_per_call": round(us, 3)})

    for B in (1, 8, 64):
        N = 144
        s = -np.sort(rng.exponential(2.0, (B, N)).astype(np.float32), axis=1)       # candidates' scores, descending
        u_at, c_at = ctypes.c_double(), ctypes.c_double()
        work = np.empty(2 * N, np.float64)
        args = (_p(s), B, N, _p(S_D), _p(S_T), M, N_table, L, n0, 0.35, ctypes.byref(u_at), ctypes.byref(c_at), _p(work))
        timed(f"tva_cast_breadth_prune B={B} N={N}", lambda: lib.tva_cast_breadth_prune(*args))
        N_tot, m = 145, 72
        ts = -rng.exponential(3.0, (B, N_tot)).astype(np.float32)
        work2 = np.empty(B * N_tot + 2 * m, np.float64)
        args2 = (_p(ts), B, N_tot, _p(S_T), M, N_table, L, n0, m, 0.3, _p(work2))
        timed(f"tva_cast_rerank_count B={B} N_tot={N_tot} m={m}", lambda: lib.tva_cast_rerank_count(*args2))
    n, keep = 145, 72
    parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)], np.int32)
    score = np.zeros(n, np.float32)
    for i in range(1, n):
        score[i] = score[parent[i]] - rng.exponential(1.0)
    old, newp, work3 = np.empty(keep, np.int32), np.empty(keep, np.int32), np.empty(n, np.int32)
    args3 = (_p(score), _p(parent), n, keep, _p(old), _p(newp), _p(work3))
    timed(f"tva_cast_select_subtree n={n} keep={keep}", lambda: lib.tva_cast_select_subtree(*args3))
    timed("tva_cast_select_context (the ctypes call alone, nearly)", lambda: lib.tva_cast_select_context(700, L, M))
    for line in out:
        print(json.dumps(line), flush=True)
    return 0


if __name__ == "__main__":
    import sys
    sys.exit(_bench())
