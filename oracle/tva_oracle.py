"""ctypes front end of the CPU oracle (``tva_oracle.c``).  TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's ``cpu_baseline`` leg import
this module.  It imports nothing from the product package and takes plain
numpy arrays (any object with the workload's attribute names works).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tva_oracle.c")
_LIB = os.path.join(_HERE, "libtva_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-std=c11", "-shared", "-fPIC",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Problem(ctypes.Structure):
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("scale", ctypes.c_double),
        ("cu_T", ctypes.c_void_p), ("L", ctypes.c_void_p), ("parent", ctypes.c_void_p),
        ("q", ctypes.c_void_p), ("k_tree", ctypes.c_void_p), ("v_tree", ctypes.c_void_p),
        ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
        ("cu_L", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("key_lo", ctypes.c_int64), ("key_hi", ctypes.c_int64),
    ]


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.tvo_num_threads.restype = ctypes.c_int
        lib.tvo_set_num_threads.argtypes = [ctypes.c_int]
        lib.tvo_ancestor_mask.restype = ctypes.c_int64
        lib.tvo_ancestor_mask.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32,
                                          ctypes.c_int32, ctypes.c_void_p]
        lib.tvo_attention.restype = ctypes.c_int
        lib.tvo_attention.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_void_p]
        lib.tvo_attention_rows.restype = ctypes.c_int
        lib.tvo_attention_rows.argtypes = [ctypes.POINTER(_Problem), ctypes.c_void_p, ctypes.c_int64,
                                           ctypes.c_void_p, ctypes.c_void_p]
        lib.tvo_merge_splits.restype = None
        lib.tvo_merge_splits.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                         ctypes.c_int32, ctypes.c_int64, ctypes.c_int32,
                                         ctypes.c_void_p, ctypes.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().tvo_num_threads())


def set_num_threads(n: int) -> None:
    _load().tvo_set_num_threads(int(n))


def _c(a: np.ndarray, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def check_trees(parent: np.ndarray, cu_T: np.ndarray) -> None:
    """Raise ValueError unless every parent is -1 or an earlier node of its tree."""
    parent = np.asarray(parent)
    cu_T = np.asarray(cu_T)
    for b in range(len(cu_T) - 1):
        p = parent[cu_T[b]:cu_T[b + 1]]
        idx = np.arange(len(p))
        if np.any(p < -1) or np.any(p >= idx):
            raise ValueError(f"tree {b}: parent array is not topological")


def ancestor_mask(parent: np.ndarray, cu_T: np.ndarray, words: Optional[int] = None) -> np.ndarray:
    """uint64 [sum_T, W] ancestor-or-self bitmasks by walking parent pointers."""
    parent = _c(parent, np.int32)
    cu_T = _c(cu_T, np.int32)
    B = len(cu_T) - 1
    max_T = int(np.max(np.diff(cu_T))) if B else 0
    W = int(words) if words is not None else max(1, (max_T + 63) // 64)
    mask = np.zeros((int(cu_T[-1]) if B else 0, W), dtype=np.uint64)
    bad = _load().tvo_ancestor_mask(_ptr(parent), _ptr(cu_T), B, W, _ptr(mask))
    if bad:
        raise ValueError(f"node {bad - 1}: parent is not in [-1, i-1]")
    return mask


def _problem(w, key_range: Optional[Tuple[int, int]]):
    keep = dict(
        cu_T=_c(w.cu_T, np.int32), L=_c(w.L, np.int32), parent=_c(w.parent, np.int32),
        q=_c(w.q, np.uint16), k_tree=_c(w.k_tree, np.uint16), v_tree=_c(w.v_tree, np.uint16),
        k_cache=_c(w.k_cache, np.uint16), v_cache=_c(w.v_cache, np.uint16),
    )
    check_trees(keep["parent"], keep["cu_T"])
    paged = getattr(w, "page_table", None) is not None
    if paged:
        keep["page_table"] = _c(w.page_table, np.int32)
        keep["cu_L"] = None
    else:
        keep["cu_L"] = _c(w.cu_L, np.int32)
        keep["page_table"] = None
    p = _Problem()
    p.B, p.Hq, p.Hkv, p.D = int(w.B), int(w.Hq), int(w.Hkv), int(w.D)
    p.scale = float(np.float32(w.scale))  # the caller's fp32 scale, widened exactly
    for name, arr in keep.items():
        setattr(p, name, _ptr(arr))
    p.page_size = int(w.page_size) if paged else 0
    p.max_pages = int(w.page_table.shape[1]) if paged else 0
    p.key_lo, p.key_hi = (0, -1) if key_range is None else (int(key_range[0]), int(key_range[1]))
    return p, keep


def tree_verify_attn(w, rows: Optional[Sequence[Tuple[int, int, int]]] = None,
                     key_range: Optional[Tuple[int, int]] = None):
    """Reference output.  Without `rows`: (out float64 [sum_T,Hq,D], lse float64
    [sum_T,Hq]).  With `rows` = [(b, node, head), ...]: (out [n,D], lse [n]).
    `key_range` = (lo, hi) restricts attention to keys lo <= k < hi of each
    sequence's concatenated [cache; tree] key list (hi < 0: unbounded)."""
    lib = _load()
    p, keep = _problem(w, key_range)
    sum_T = int(keep["cu_T"][-1]) if w.B else 0
    if rows is None:
        out = np.zeros((sum_T, w.Hq, w.D), dtype=np.float64)
        lse = np.zeros((sum_T, w.Hq), dtype=np.float64)
        rc = lib.tvo_attention(ctypes.byref(p), _ptr(out), _ptr(lse))
    else:
        r = _c(np.asarray(rows).reshape(-1, 3), np.int32)
        for b, i, h in r:
            if not (0 <= b < w.B and 0 <= h < w.Hq and 0 <= i < keep["cu_T"][b + 1] - keep["cu_T"][b]):
                raise ValueError(f"row {(b, i, h)} out of range")
        out = np.zeros((len(r), w.D), dtype=np.float64)
        lse = np.zeros((len(r),), dtype=np.float64)
        rc = lib.tvo_attention_rows(ctypes.byref(p), _ptr(r), len(r), _ptr(out), _ptr(lse))
    if rc:
        raise MemoryError("oracle allocation failed")
    return out, lse


def merge_splits(part_out: np.ndarray, part_lse: np.ndarray,
                 n_splits_row: Optional[np.ndarray] = None):
    """Merge partial results over disjoint key subsets: part_out [S, n, D],
    part_lse [S, n] -> (out [n, D], lse [n])."""
    po = _c(part_out, np.float64)
    pl = _c(part_lse, np.float64)
    S, n, D = po.shape
    ns = None if n_splits_row is None else _c(n_splits_row, np.int32)
    out = np.zeros((n, D), dtype=np.float64)
    lse = np.zeros((n,), dtype=np.float64)
    _load().tvo_merge_splits(_ptr(po), _ptr(pl), _ptr(ns), S, n, D, _ptr(out), _ptr(lse))
    return out, lse
