"""Device plumbing for the tests, the smoke check and the benchmark: copies a host
workload into torch device tensors and calls the library through the binding.
No arithmetic of the method happens here."""
from __future__ import annotations

import dataclasses
from typing import Optional

import numpy as np

from . import binding


@dataclasses.dataclass
class DeviceWorkload:
    w: object            # the host workload (shapes only are used after upload)
    q: object
    k_tree: object
    v_tree: object
    k_cache: object
    v_cache: object
    cu_T: object
    L: object
    parent: object
    cu_L: Optional[object]
    page_table: Optional[object]


def _dev(a: np.ndarray, device):
    import torch
    if a.dtype == np.uint16:
        a = a.view(np.int16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_device(w, device="cuda:0") -> DeviceWorkload:
    return DeviceWorkload(
        w=w, q=_dev(w.q, device), k_tree=_dev(w.k_tree, device), v_tree=_dev(w.v_tree, device),
        k_cache=_dev(w.k_cache, device), v_cache=_dev(w.v_cache, device),
        cu_T=_dev(w.cu_T, device), L=_dev(w.L, device), parent=_dev(w.parent, device),
        cu_L=None if w.cu_L is None else _dev(w.cu_L, device),
        page_table=None if w.page_table is None else _dev(w.page_table, device))


def build_mask(dw: DeviceWorkload, err_flag=None, stream=None):
    return binding.build_ancestor_mask(dw.parent, dw.cu_T, max(1, dw.w.max_T), err_flag=err_flag, stream=stream)


def attention(dw: DeviceWorkload, mask, num_splits: int = 0, max_L: Optional[int] = None, strides=(0, 0, 0),
              out=None, lse=None, workspace=None, stream=None, k_scale: float = 1.0, v_scale: float = 1.0,
              sum_L: int = 0, plan_shape: int = 0, L_host=None):
    """mask=None: the parent arrays are passed instead and the kernel derives the ancestor sets.
    A workload whose K/V are uint8 is taken as E4M3 bytes with the two scales."""
    import torch
    w = dw.w
    fp8 = dw.k_cache.dtype == torch.uint8
    return binding.tree_verify_attn(
        dw.q, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, mask, dw.cu_T, dw.L,
        max_T=w.max_T, max_L=w.max_L if max_L is None else max_L, scale=w.scale, cu_L=dw.cu_L,
        page_table=dw.page_table, page_size=w.page_size, strides=strides, num_splits=num_splits,
        out=out, lse=lse, workspace=workspace, stream=stream, parent=dw.parent if mask is None else None,
        kv_fp8=fp8, k_scale=k_scale, v_scale=v_scale, sum_L=sum_L, plan_shape=plan_shape, L_host=L_host)


def run_path(dw: DeviceWorkload, num_splits: int = 0, sum_L: int = 0, plan_shape: int = 0, L_host=None):
    """The whole hot path once: ancestor masks, split-KV attention, merge."""
    mask = build_mask(dw)
    out, lse = attention(dw, mask, num_splits=num_splits, sum_L=sum_L, plan_shape=plan_shape, L_host=L_host)
    return mask, out, lse
