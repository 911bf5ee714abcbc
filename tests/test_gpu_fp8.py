"""GPU parity of the attention on an 8-bit floating point (E4M3) KV cache against the CPU oracle that
decodes the same bytes: same tolerances as the bf16 path (the kernel widens the bytes exactly and then
runs the bf16 arithmetic)."""
import dataclasses

import numpy as np
import pytest

from oracle import fp8_oracle as f8
from paper_2510_26577_amd import workloads as wl

pytestmark = pytest.mark.gpu

TOL_O = 2e-3
TOL_LSE = 1e-4


@pytest.fixture(scope="module")
def gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_26577_amd import binding, device
    binding.load_library()
    return device


def say(msg):
    print(msg, flush=True)


def check(gpu, w8, ks, vs, num_splits=0, derive=False, label="", plan_shape=0, hints=False):
    """hints: the host's copy of the cache lengths and their sum are passed, as the benchmark does."""
    import torch
    say(f"[case] fp8 {label} B={w8.B} T={list(w8.T[:6])} L={list(w8.L[:6])} paged={w8.paged} splits={num_splits} hints={hints}")
    dw = gpu.to_device(w8)
    mask = None if derive else gpu.build_mask(dw)
    lens = np.ascontiguousarray(w8.L, dtype=np.int32)
    out, lse = gpu.attention(dw, mask, num_splits=num_splits, k_scale=ks, v_scale=vs, plan_shape=plan_shape,
                             sum_L=int(lens.sum()) if hints else 0, L_host=lens if hints else None)
    torch.cuda.synchronize()
    ro, rl = f8.tree_verify_attn_fp8(w8, ks, vs)
    o, l = out.cpu().numpy().astype(np.float64), lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    eo = np.abs(o - ro).max() if o.size else 0.0
    el = np.abs(l - rl).max() if l.size else 0.0
    say(f"        max|dO|={eo:.3e} max|dLSE|={el:.3e}")
    assert eo <= TOL_O and el <= TOL_LSE
    return eo, el


@pytest.mark.parametrize("variant", [0, 1, 2, 4, 5])
@pytest.mark.parametrize("page", [0, 16])
def test_fp8_shapes_dense_and_paged(gpu, variant, page):
    w = wl.random_workload(1300 + page, 4, 8, 2, 128, [900, 130, 0, 517], [70, 33, 8, 64], max_depth=10, page_size=page)
    w8, ks, vs = wl.to_fp8_kv(w)
    for splits in (0, 3):
        check(gpu, w8, ks, vs, num_splits=splits, label=f"shape {variant}", plan_shape=variant)
    check(gpu, w8, ks, vs, num_splits=2, derive=True, label=f"shape {variant}, masks derived", plan_shape=variant)


def test_every_code_is_widened_exactly(gpu):
    """K and V made of all 254 non-NaN codes (each head-dimension lane sees each code): a wrong exponent bias,
    a mishandled subnormal or a swapped byte order inside a dword shows here."""
    w = wl.random_workload(1310, 1, 4, 1, 128, [254], [5], max_depth=3)
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    k8 = np.empty((254, 1, 128), np.uint8)
    v8 = np.empty((254, 1, 128), np.uint8)
    for d in range(128):
        k8[:, 0, d] = np.roll(codes, 7 * d)
        v8[:, 0, d] = np.roll(codes, 11 * d + 3)
    rng = np.random.Generator(np.random.PCG64(5))
    kt = codes[rng.integers(0, 254, (5, 1, 128))]
    vt = codes[rng.integers(0, 254, (5, 1, 128))]
    w8 = dataclasses.replace(w, k_cache=k8, v_cache=v8, k_tree=kt, v_tree=vt)
    # scales small enough that the scores stay moderate: |k| <= 448
    check(gpu, w8, 1.0 / 4096, 1.0 / 128, label="all codes")


@pytest.mark.parametrize("hints", [False, True])
@pytest.mark.parametrize("B,L,T", [(1, 2048, 60), (16, 2048, 16), (8, 2048, 60), (40, 700, 8), (64, 900, 8)])
def test_fp8_benchmark_like_shapes(gpu, B, L, T, hints):
    rng = np.random.Generator(np.random.PCG64(B + L + T))
    Ls = rng.integers(L // 2, L + 1, B)
    Ls[0] = L
    w = wl.random_workload(1320 + B, B, 32, 8, 128, Ls, T, max_depth=8)
    w8, ks, vs = wl.to_fp8_kv(w)
    check(gpu, w8, ks, vs, label="benchmark-like", hints=hints)


def test_fp8_rejects_head_dimension_64(gpu):
    import torch
    from paper_2510_26577_amd import binding
    w = wl.random_workload(1330, 1, 4, 2, 64, [40], [5])
    w8, ks, vs = wl.to_fp8_kv(w)
    dw = gpu.to_device(w8)
    with pytest.raises(binding.TvaError):
        gpu.attention(dw, None, k_scale=ks, v_scale=vs)


def _rows_in_cache(w8, page_size, rng):
    """Re-stores an fp8 workload with the tree's K/V bytes behind each sequence's committed tokens."""
    B, Hkv, D = w8.B, w8.Hkv, w8.D
    tot = w8.L.astype(np.int64) + w8.T.astype(np.int64)
    rows = lambda b, cache, tree: np.concatenate([cache[w8.cu_L[b]:w8.cu_L[b] + w8.L[b]], tree[w8.cu_T[b]:w8.cu_T[b + 1]]])
    if page_size == 0:
        cu = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
        return (np.concatenate([rows(b, w8.k_cache, w8.k_tree) for b in range(B)]),
                np.concatenate([rows(b, w8.v_cache, w8.v_tree) for b in range(B)]), cu, None)
    max_pages = int((tot.max() + page_size - 1) // page_size) + 1
    table = rng.permutation(B * max_pages).reshape(B, max_pages).astype(np.int32)
    k = np.full((B * max_pages, page_size, Hkv, D), 0x7E, np.uint8)      # 448 everywhere a stray read would land
    v = k.copy()
    for b in range(B):
        kr, vr = rows(b, w8.k_cache, w8.k_tree), rows(b, w8.v_cache, w8.v_tree)
        for t in range(int(tot[b])):
            k[table[b, t // page_size], t % page_size] = kr[t]
            v[table[b, t // page_size], t % page_size] = vr[t]
    return k, v, None, table


@pytest.mark.parametrize("page_size", [0, 16])
@pytest.mark.parametrize("variant", [0, 1, 4, 5])
def test_fp8_tree_rows_in_the_cache_and_query_subsets(gpu, page_size, variant):
    """The other input variants on the 8-bit path: tree K/V stored in the cache (k_tree = NULL), and only the
    newest nodes of each tree as queries (cu_Q); both against the oracle on the same bytes."""
    import torch
    from paper_2510_26577_amd import binding
    rng = np.random.Generator(np.random.PCG64(1400 + page_size))
    w = wl.random_workload(1400 + page_size, 4, 8, 2, 128, [300, 64, 0, 129], [70, 33, 8, 128], max_depth=12)
    w8, ks, vs = wl.to_fp8_kv(w)
    ro, rl = f8.tree_verify_attn_fp8(w8, ks, vs)
    k, v, cu, table = _rows_in_cache(w8, page_size, rng)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    q, cu_T, L, parent = dev(w8.q.view(np.int16)), dev(w8.cu_T), dev(w8.L.astype(np.int32)), dev(w8.parent)
    kd, vd, cud, tabd = dev(k), dev(v), dev(cu), dev(table)
    say(f"[case] fp8 tree rows in cache, page_size={page_size} variant={variant}")
    for splits in (0, 3):
        out, lse = binding.tree_verify_attn(q, None, None, kd, vd, None, cu_T, L, max_T=w8.max_T, max_L=w8.max_L,
                                            scale=w8.scale, cu_L=cud, page_table=tabd, page_size=page_size,
                                            num_splits=splits, parent=parent, kv_fp8=True, k_scale=ks, v_scale=vs,
                                            plan_shape=variant)
        torch.cuda.synchronize()
        assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
        assert np.abs(lse.cpu().numpy().astype(np.float64) - rl).max() <= TOL_LSE
    Tq = np.array([12, 33, 1, 60])
    cu_Q = np.concatenate([[0], np.cumsum(Tq)]).astype(np.int32)
    sel = np.concatenate([np.arange(w8.cu_T[b + 1] - Tq[b], w8.cu_T[b + 1]) for b in range(w8.B)]).astype(np.int64)
    say(f"[case] fp8 query subset, page_size={page_size} variant={variant}")
    out, lse = binding.tree_verify_attn(q[torch.from_numpy(sel).cuda()].contiguous(), None, None, kd, vd, None, cu_T, L,
                                        max_T=w8.max_T, max_L=w8.max_L, scale=w8.scale, cu_L=cud, page_table=tabd,
                                        page_size=page_size, parent=parent, cu_Q=dev(cu_Q), max_Q=int(Tq.max()),
                                        sum_T=w8.sum_T, kv_fp8=True, k_scale=ks, v_scale=vs, plan_shape=variant)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy().astype(np.float64) - ro[sel]).max() <= TOL_O
    assert np.abs(lse.cpu().numpy().astype(np.float64) - rl[sel]).max() <= TOL_LSE
