"""GPU test of tva_tree_verify_attn_static, the entry point that allocates nothing (the KV splits'
partial results go to a device array inside the library): its output must equal
tva_tree_verify_attn's on the same inputs, on two calls in a row, the second with a smaller input
that reuses the front of the array the first call filled."""
import ctypes
import sys

import numpy as np
import pytest

from paper_2510_26577_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL_O, TOL_LSE = 2e-3, 1e-4


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def _both(binding, device, w, num_splits, page_size=0):
    """(out, lse) of the workspace entry point and of the static one, same inputs."""
    import torch
    dw = device.to_device(w)
    res = []
    for static in (False, True):
        out = torch.full((w.sum_T, w.Hq, w.D), float("nan"), dtype=torch.float32, device="cuda:0")
        lse = torch.full((w.sum_T, w.Hq), float("nan"), dtype=torch.float32, device="cuda:0")
        args = binding.make_args(q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                                 anc_mask=None, parent=dw.parent, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L,
                                 scale=w.scale, cu_L=dw.cu_L, page_table=dw.page_table, page_size=w.page_size,
                                 num_splits=num_splits, out=out, lse=lse)
        need = binding.workspace_bytes(args)
        assert 0 < need <= binding.STATIC_SCRATCH_BYTES, need
        if static:
            binding.tree_verify_attn_static_raw(args)          # args.workspace stays NULL
        else:
            ws = torch.empty(need // 4, dtype=torch.float32, device="cuda:0")
            args.workspace, args.workspace_bytes = ws.data_ptr(), need
            binding.tree_verify_attn_raw(args)
        torch.cuda.synchronize()
        res.append((out.cpu().numpy(), lse.cpu().numpy()))
    return res


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import tva_oracle as orc
    from paper_2510_26577_amd import binding, device
    binding.load_library()
    cases = [
        ("first: 3 ragged sequences, 5 splits", wl.random_workload(4100, 3, 16, 4, 128, [1500, 700, 64], [72, 40, 9], max_depth=10), 5),
        ("second, smaller: 2 sequences, 3 splits", wl.random_workload(4101, 2, 8, 2, 128, [400, 130], [33, 8], max_depth=6), 3),
        ("third, paged", wl.random_workload(4102, 2, 8, 2, 128, [517, 64], [40, 64], page_size=16), 2),
    ]
    for label, w, splits in cases:
        say(f"[case] static scratch, {label}: B={w.B} T={list(w.T)} L={list(w.L)} splits={splits}")
        (o_ws, l_ws), (o_st, l_st) = _both(binding, device, w, splits)
        assert np.isfinite(o_st).all() and np.isfinite(l_st).all()
        # same kernels, same launch plan, no atomics: the two entry points agree to the bit
        assert np.array_equal(o_ws, o_st) and np.array_equal(l_ws, l_st)
        ro, rl = orc.tree_verify_attn(w)
        eo, el = np.abs(o_st - ro).max(), np.abs(l_st - rl).max()
        say(f"        vs oracle max|dO|={eo:.3e} max|dLSE|={el:.3e}")
        assert eo <= TOL_O and el <= TOL_LSE
    # a plan that needs more than the array holds is refused and queues nothing
    big = wl.random_workload(4103, 8, 64, 8, 128, [4096] * 8, [128] * 8, max_depth=12)
    dw = device.to_device(big)
    out = torch.zeros((big.sum_T, big.Hq, big.D), dtype=torch.float32, device="cuda:0")
    lse = torch.zeros((big.sum_T, big.Hq), dtype=torch.float32, device="cuda:0")
    args = binding.make_args(q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                             anc_mask=None, parent=dw.parent, cu_T=dw.cu_T, L=dw.L, max_T=big.max_T, max_L=big.max_L,
                             scale=big.scale, cu_L=dw.cu_L, num_splits=4, out=out, lse=lse)
    assert binding.workspace_bytes(args) > binding.STATIC_SCRATCH_BYTES
    rc = binding.load_library().tva_tree_verify_attn_static(ctypes.byref(args), None)
    assert rc == -3
    torch.cuda.synchronize()
    assert not out.any().item()
