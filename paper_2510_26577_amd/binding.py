"""Thin ctypes binding of libtva (argument marshalling only).

Every step of the path runs in the HIP kernels of ``libtva.so``; this module
turns torch tensors into raw device pointers and fills the C argument struct
declared in ``include/tva.h``.  torch is used for device memory and streams
only.  There is no CPU fallback: if the library is missing, loading raises.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
LIB_PATH = os.path.join(_HERE, "libtva.so")
TIMELINE_LIB_PATH = os.path.join(_HERE, "libtva_timeline.so")  # the same sources with time stamps in the kernels
SRC_PATH = os.path.join(_HERE, "csrc", "tva.hip")
CAST_SRC_PATH = os.path.join(_HERE, "csrc", "cast.cpp")  # host part: tree-size selection
VERIFY_SRC_PATH = os.path.join(_HERE, "csrc", "verify.hip")  # acceptance + commit kernels
DRAFT_SRC_PATH = os.path.join(_HERE, "csrc", "draft.hip")    # draft-tree expansion + subtree kernels
INCLUDE_DIR = os.path.join(_ROOT, "include")

TVA_OK = 0
TVA_MAX_TREE = 128
EXPECTED_VERSION = 7
# tva_shape (include/tva.h): workgroup shapes a caller may name in tva_args.plan_shape
SHAPE_AUTO, SHAPE_R32_W2, SHAPE_R64_W4, SHAPE_R64_W4_DEEP, SHAPE_R128_W8, SHAPE_R256_W8 = range(6)
SHAPES = (SHAPE_R32_W2, SHAPE_R64_W4, SHAPE_R64_W4_DEEP, SHAPE_R128_W8, SHAPE_R256_W8)
STATIC_SCRATCH_BYTES = 32 << 20

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False, timeline: bool = False) -> str:
    """Compile csrc/tva.hip, csrc/verify.hip and csrc/draft.hip (gfx950 kernels + their C ABI) and csrc/cast.cpp
    (host logic) into libtva.so (in-tree); timeline=True: the instrumented build libtva_timeline.so
    (paper_2510_26577_amd/timeline.py) instead."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = TIMELINE_LIB_PATH if timeline else LIB_PATH
    cmd = [hipcc, *HIPCC_FLAGS, *(["-DTVA_TIMELINE"] if timeline else []), "-I", INCLUDE_DIR, "-shared", "-fPIC", "-o", out,
           SRC_PATH, VERIFY_SRC_PATH, DRAFT_SRC_PATH, CAST_SRC_PATH]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    lines = [l for l in res.stdout.splitlines() if "is not a recognized feature" not in l]
    if verbose or res.returncode:
        print("\n".join(lines))
    if res.returncode:
        raise RuntimeError(f"hipcc failed building {os.path.basename(out)}")
    return out


class TvaArgs(ctypes.Structure):
    """Mirror of `struct tva_args`."""
    _fields_ = [
        ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32), ("D", ctypes.c_int32),
        ("sum_T", ctypes.c_int32), ("max_T", ctypes.c_int32), ("mask_words", ctypes.c_int32),
        ("max_L", ctypes.c_int32), ("scale", ctypes.c_float),
        ("cu_T", ctypes.c_void_p), ("L", ctypes.c_void_p),
        ("q", ctypes.c_void_p), ("k_tree", ctypes.c_void_p), ("v_tree", ctypes.c_void_p),
        ("anc_mask", ctypes.c_void_p),
        ("k_cache", ctypes.c_void_p), ("v_cache", ctypes.c_void_p),
        ("cu_L", ctypes.c_void_p), ("page_table", ctypes.c_void_p),
        ("page_size", ctypes.c_int32), ("max_pages", ctypes.c_int32),
        ("stride_page", ctypes.c_int64), ("stride_tok", ctypes.c_int64), ("stride_head", ctypes.c_int64),
        ("out", ctypes.c_void_p), ("lse", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
        ("num_splits", ctypes.c_int32),
        ("parent", ctypes.c_void_p),
        ("cu_Q", ctypes.c_void_p), ("sum_Q", ctypes.c_int32), ("max_Q", ctypes.c_int32),
        ("kv_fp8", ctypes.c_int32), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float),
        ("sum_L", ctypes.c_int64),
        ("plan_shape", ctypes.c_int32),
        ("L_host", ctypes.c_void_p),
    ]


EXPORTS = ("tva_build_ancestor_mask", "tva_build_ancestor_mask_host", "tva_workspace_bytes", "tva_plan_splits", "tva_plan_chunk_keys", "tva_plan_workgroup_rows", "tva_plan_slot_sequences",
           "tva_tree_verify_attn", "tva_tree_verify_attn_static", "tva_static_scratch_bytes", "tva_tree_verify_attn_splits", "tva_merge_splits", "tva_strerror", "tva_version", "tva_sizeof_args", "tva_timeline_read")
# entry points of include/tva_verify.h (bound in verify.py)
DRAFT_EXPORTS = ("tva_expand_workspace_bytes", "tva_expand_layer", "tva_sizeof_expand_args", "tva_tree_select_subtree",
                 "tva_tree_rerank_count", "tva_rerank_workspace_bytes",
                 "tva_layer_breadth_count")
VERIFY_EXPORTS = ("tva_accept_greedy", "tva_accept_sampling", "tva_accept_sampling_wait_bound_test", "tva_sample_workspace_bytes", "tva_sample_workspace_bytes_rows", "tva_sizeof_sample_args", "tva_commit_path",
                  "tva_sizeof_commit_args")
# host entry points of include/tva_cast.h (bound in cast.py)
CAST_EXPORTS = ("tva_cast_select_context", "tva_cast_select_max_valid_index", "tva_cast_layer_utility",
                "tva_cast_layer_cost", "tva_cast_breadth_prune", "tva_cast_depth_bytes", "tva_cast_depth_init",
                "tva_cast_depth_alpha", "tva_cast_depth_should_expand", "tva_cast_depth_update",
                "tva_cast_expansion_plan", "tva_cast_rerank_count", "tva_cast_select_subtree")

_lib = None


def use_timeline_library() -> None:
    """Profiling tools: make this process load the instrumented build.  Before the first load only."""
    global LIB_PATH
    if _lib is not None:
        raise RuntimeError("libtva is already loaded")
    LIB_PATH = TIMELINE_LIB_PATH


def load_library():
    """Load libtva.so; raises if it is absent (there is no fallback path)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    # torch first: it brings the HIP runtime the process shares.  Loaded the other way round, libtva.so
    # pulls in the system's copy, torch then loads its own, and the second one finds no device.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    lib.tva_version.restype = ctypes.c_int
    lib.tva_strerror.restype = ctypes.c_char_p
    lib.tva_strerror.argtypes = [ctypes.c_int]
    lib.tva_build_ancestor_mask.restype = ctypes.c_int
    lib.tva_build_ancestor_mask.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                            ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.tva_build_ancestor_mask_host.restype = ctypes.c_int
    lib.tva_build_ancestor_mask_host.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                                 ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
    lib.tva_workspace_bytes.restype = ctypes.c_size_t
    lib.tva_workspace_bytes.argtypes = [ctypes.POINTER(TvaArgs)]
    lib.tva_plan_splits.restype = ctypes.c_int32
    lib.tva_plan_splits.argtypes = [ctypes.POINTER(TvaArgs)]
    lib.tva_plan_chunk_keys.restype = ctypes.c_int32
    lib.tva_plan_chunk_keys.argtypes = [ctypes.POINTER(TvaArgs)]
    lib.tva_plan_slot_sequences.restype = ctypes.c_int32
    lib.tva_plan_slot_sequences.argtypes = [ctypes.POINTER(TvaArgs), ctypes.POINTER(ctypes.c_int32)]
    lib.tva_plan_workgroup_rows.restype = ctypes.c_int32
    lib.tva_plan_workgroup_rows.argtypes = [ctypes.POINTER(TvaArgs)]
    lib.tva_tree_verify_attn.restype = ctypes.c_int
    lib.tva_tree_verify_attn.argtypes = [ctypes.POINTER(TvaArgs), ctypes.c_void_p]
    lib.tva_tree_verify_attn_static.restype = ctypes.c_int
    lib.tva_tree_verify_attn_static.argtypes = [ctypes.POINTER(TvaArgs), ctypes.c_void_p]
    lib.tva_static_scratch_bytes.restype = ctypes.c_size_t
    lib.tva_tree_verify_attn_splits.restype = ctypes.c_int
    lib.tva_tree_verify_attn_splits.argtypes = [ctypes.POINTER(TvaArgs), ctypes.c_void_p]
    lib.tva_merge_splits.restype = ctypes.c_int
    lib.tva_merge_splits.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64,
                                     ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    lib.tva_sizeof_args.restype = ctypes.c_size_t
    lib.tva_timeline_read.restype = ctypes.c_int
    lib.tva_timeline_read.argtypes = [ctypes.c_void_p, ctypes.c_int32]
    if lib.tva_version() != EXPECTED_VERSION or lib.tva_sizeof_args() != ctypes.sizeof(TvaArgs):
        raise RuntimeError("libtva.so is stale: rebuild it")
    _lib = lib
    return lib


class TvaError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"libtva: {load_library().tva_strerror(code).decode()} ({code})")


def _check(code: int) -> None:
    if code != TVA_OK:
        raise TvaError(code)


def _stream_ptr(stream) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


def _p(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def build_ancestor_mask_host(parent, cu_T, max_T: int):
    """numpy int32 arrays on the host -> (uint64 mask [sum_T, W], status, bad_node).  Validation variant:
    status is TVA_OK or TVA_BAD_TREE (-5), bad_node the first offending global node index or -1."""
    import numpy as np
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    cu_T = np.ascontiguousarray(cu_T, dtype=np.int32)
    B = len(cu_T) - 1
    W = max(1, (int(max_T) + 63) // 64)
    mask = np.zeros((int(cu_T[-1]), W), np.uint64)
    bad = ctypes.c_int32(-1)
    rc = load_library().tva_build_ancestor_mask_host(parent.ctypes.data, cu_T.ctypes.data, B, int(max_T), W,
                                                     mask.ctypes.data, ctypes.byref(bad))
    if rc not in (TVA_OK, -5):
        raise TvaError(rc)
    return mask, rc, bad.value


def build_ancestor_mask(parent, cu_T, max_T: int, mask=None, err_flag=None, stream=None):
    """parent int32 [sum_T], cu_T int32 [B+1] (device) -> mask int64 [sum_T, W]
    holding the uint64 bit patterns.  `err_flag` (int32[1], zeroed by the
    caller) receives 1 + index of the first malformed node, asynchronously."""
    import torch
    lib = load_library()
    B = cu_T.numel() - 1
    W = max(1, (int(max_T) + 63) // 64)
    if mask is None:
        mask = torch.empty((parent.numel(), W), dtype=torch.int64, device=parent.device)
    else:
        W = mask.shape[1]
    _check(lib.tva_build_ancestor_mask(_p(parent), _p(cu_T), B, int(max_T), W, _p(mask), _p(err_flag),
                                       _stream_ptr(stream)))
    return mask


def make_args(*, q, k_tree, v_tree, k_cache, v_cache, anc_mask, cu_T, L, max_T: int, max_L: int,
              scale: float, cu_L=None, page_table=None, page_size: int = 0, strides=(0, 0, 0),
              num_splits: int = 0, out=None, lse=None, workspace=None, parent=None, cu_Q=None, max_Q: int = 0,
              sum_T: Optional[int] = None, kv_fp8: bool = False, k_scale: float = 1.0, v_scale: float = 1.0,
              sum_L: int = 0, plan_shape: int = 0, L_host=None) -> TvaArgs:
    """Fill `tva_args` from tensors (q [sum_T,Hq,D], k_tree [sum_T,Hkv,D], ...).  With cu_Q (queries =
    the last nodes of each tree) q has sum_Q rows and sum_T comes from k_tree or the sum_T argument.
    L_host: the cache lengths as a host array (numpy int32 [B]), the optional placement hint."""
    a = TvaArgs()
    a.B = cu_T.numel() - 1
    a.sum_T, a.Hq, a.D = int(q.shape[0]), int(q.shape[1]), int(q.shape[2])
    if cu_Q is not None:
        a.sum_Q, a.max_Q = int(q.shape[0]), int(max_Q)
        a.sum_T = int(sum_T) if sum_T is not None else int(k_tree.shape[0])
    a.cu_Q = _p(cu_Q)
    a.Hkv = int(k_tree.shape[1]) if k_tree is not None else int(k_cache.shape[-2])
    a.max_T, a.max_L = int(max_T), int(max_L)
    a.mask_words = int(anc_mask.shape[1]) if anc_mask is not None else max(1, (int(max_T) + 63) // 64)
    a.scale = float(scale)
    a.cu_T, a.L = _p(cu_T), _p(L)
    a.q, a.k_tree, a.v_tree, a.anc_mask = _p(q), _p(k_tree), _p(v_tree), _p(anc_mask)
    a.k_cache, a.v_cache = _p(k_cache), _p(v_cache)
    a.cu_L, a.page_table = _p(cu_L), _p(page_table)
    a.page_size = int(page_size)
    a.max_pages = int(page_table.shape[1]) if page_table is not None else 0
    a.stride_page, a.stride_tok, a.stride_head = (int(s) for s in strides)
    a.out, a.lse = _p(out), _p(lse)
    a.workspace = _p(workspace)
    a.workspace_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    a.num_splits = int(num_splits)
    a.parent = _p(parent)
    a.kv_fp8, a.k_scale, a.v_scale = int(bool(kv_fp8)), float(k_scale), float(v_scale)
    a.sum_L = int(sum_L)
    a.plan_shape = int(plan_shape)
    if L_host is not None:
        import numpy as np
        L_host = np.ascontiguousarray(L_host, dtype=np.int32)
        assert L_host.shape == (a.B,)
        a.L_host = L_host.ctypes.data
    # the struct holds raw addresses: keep the tensors alive as long as it lives
    a._keep = (q, k_tree, v_tree, k_cache, v_cache, anc_mask, cu_T, L, cu_L, page_table, out, lse, workspace, parent, cu_Q, L_host)
    return a


def workspace_bytes(args: TvaArgs) -> int:
    n = load_library().tva_workspace_bytes(ctypes.byref(args))
    if n == ctypes.c_size_t(-1).value:
        raise TvaError(-1)
    return int(n)


def plan_splits(args: TvaArgs) -> int:
    n = load_library().tva_plan_splits(ctypes.byref(args))
    if n < 0:
        raise TvaError(-1)
    return int(n)


def plan_chunk_keys(args: TvaArgs) -> int:
    n = load_library().tva_plan_chunk_keys(ctypes.byref(args))
    if n < 0:
        raise TvaError(-1)
    return int(n)


def plan_slot_sequences(args: TvaArgs):
    """The sequence each workgroup slot takes (a list, empty when the sequences keep their order)."""
    out = (ctypes.c_int32 * 64)()
    n = load_library().tva_plan_slot_sequences(ctypes.byref(args), out)
    if n < 0:
        raise TvaError(-1)
    return list(out[:n])


def plan_workgroup_rows(args: TvaArgs) -> int:
    n = load_library().tva_plan_workgroup_rows(ctypes.byref(args))
    if n < 0:
        raise TvaError(-1)
    return int(n)


def tree_verify_attn_raw(args: TvaArgs, stream=None) -> None:
    """Queue the attention on `stream` with a prepared argument struct."""
    _check(load_library().tva_tree_verify_attn(ctypes.byref(args), _stream_ptr(stream)))


def tree_verify_attn_static_raw(args: TvaArgs, stream=None) -> None:
    """Queue the attention with the KV splits' partial results in the library's own device array
    (tva_tree_verify_attn_static: nothing is allocated, args.workspace is ignored)."""
    _check(load_library().tva_tree_verify_attn_static(ctypes.byref(args), _stream_ptr(stream)))


def tree_verify_attn_splits_raw(args: TvaArgs, stream=None) -> None:
    """Queue only the split-KV attention kernel (no merge) with a prepared argument struct."""
    _check(load_library().tva_tree_verify_attn_splits(ctypes.byref(args), _stream_ptr(stream)))


def tree_verify_attn(q, k_tree, v_tree, k_cache, v_cache, anc_mask, cu_T, L, *, max_T: int, max_L: int,
                     scale: float, cu_L=None, page_table=None, page_size: int = 0, strides=(0, 0, 0),
                     num_splits: int = 0, out=None, lse=None, workspace=None, stream=None, parent=None, cu_Q=None,
                     max_Q: int = 0, sum_T: Optional[int] = None, kv_fp8: bool = False, k_scale: float = 1.0,
                     v_scale: float = 1.0, sum_L: int = 0, plan_shape: int = 0, L_host=None):
    """Tree-masked verification attention.  Returns (out fp32 [sum_T,Hq,D], lse fp32 [sum_T,Hq]).
    bf16 tensors may be torch.bfloat16 or int16/uint16 bit patterns; with kv_fp8 the K/V tensors are uint8
    (E4M3 bytes) and K = k_scale * value, V = v_scale * value.  anc_mask may be None when the
    trees' parent array (int32 [sum_T]) is passed instead: the kernel then derives the masks itself."""
    import torch
    if out is None:
        out = torch.empty(q.shape, dtype=torch.float32, device=q.device)
    if lse is None:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    args = make_args(q=q, k_tree=k_tree, v_tree=v_tree, k_cache=k_cache, v_cache=v_cache, anc_mask=anc_mask,
                     cu_T=cu_T, L=L, max_T=max_T, max_L=max_L, scale=scale, cu_L=cu_L, page_table=page_table,
                     page_size=page_size, strides=strides, num_splits=num_splits, out=out, lse=lse, parent=parent,
                     cu_Q=cu_Q, max_Q=max_Q, sum_T=sum_T, kv_fp8=kv_fp8, k_scale=k_scale, v_scale=v_scale, sum_L=sum_L,
                     plan_shape=plan_shape, L_host=L_host)
    need = workspace_bytes(args)
    if need and (workspace is None or workspace.numel() * workspace.element_size() < need):
        workspace = torch.empty((need + 3) // 4, dtype=torch.float32, device=q.device)
    if workspace is not None:
        args.workspace = workspace.data_ptr()
        args.workspace_bytes = workspace.numel() * workspace.element_size()
    tree_verify_attn_raw(args, stream)
    return out, lse


def merge_splits(part_out, part_lse, out=None, lse=None, stream=None):
    """part_out fp32 [S, n, D], part_lse fp32 [S, n] -> (out [n, D], lse [n])."""
    import torch
    S, n, D = part_out.shape
    if out is None:
        out = torch.empty((n, D), dtype=torch.float32, device=part_out.device)
    if lse is None:
        lse = torch.empty((n,), dtype=torch.float32, device=part_out.device)
    _check(load_library().tva_merge_splits(_p(part_out), _p(part_lse), S, n, D, _p(out), _p(lse),
                                           _stream_ptr(stream)))
    return out, lse
