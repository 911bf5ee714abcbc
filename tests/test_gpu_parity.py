"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element, on the same seeded inputs.  Tolerances are the ones the task fixes:
max-abs 2e-3 on O, 1e-4 on LSE, ancestor masks bit-exact."""
import sys

import numpy as np
import pytest

from oracle import tva_oracle as orc
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
    binding.load_library()  # raises if the HIP library is missing: no fallback
    return device


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def check_full(device, w, num_splits=0, label="", plan_shape=0, hints=False):
    """hints: the host's copy of the cache lengths and their sum are passed, as the benchmark does."""
    import torch
    say(f"[case] {label or w.name} B={w.B} Hq={w.Hq} Hkv={w.Hkv} D={w.D} T={list(w.T[:6])} L={list(w.L[:6])} "
        f"paged={w.paged} splits={num_splits} hints={hints}")
    dw = device.to_device(w)
    lens = np.ascontiguousarray(w.L, dtype=np.int32)
    mask, out, lse = device.run_path(dw, num_splits=num_splits, plan_shape=plan_shape, sum_L=int(lens.sum()) if hints else 0,
                                     L_host=lens if hints else None)
    torch.cuda.synchronize()
    ref_mask = orc.ancestor_mask(w.parent, w.cu_T, words=mask.shape[1]) if w.sum_T else np.zeros((0, 1), np.uint64)
    assert np.array_equal(mask.cpu().numpy().view(np.uint64).reshape(ref_mask.shape), ref_mask)
    ro, rl = orc.tree_verify_attn(w)
    o = out.cpu().numpy().astype(np.float64)
    l = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    eo = np.abs(o - ro).max() if o.size else 0.0
    el = np.abs(l - rl).max() if l.size else 0.0
    say(f"        max|dO|={eo:.3e} max|dLSE|={el:.3e}")
    assert eo <= TOL_O and el <= TOL_LSE
    return eo, el


# ------------------------------------------------------------------ the five configurations
# (with the hints: the launch configuration the benchmark times; without: what a caller that passes none gets)
@pytest.mark.parametrize("hints", [True, False])
def test_config1_tiny(gpu, hints):
    check_full(gpu, wl.config1(), hints=hints)


@pytest.mark.parametrize("splits,hints", [(0, True), (0, False), (1, False), (3, False), (32, False)])
def test_config2_8b(gpu, splits, hints):
    check_full(gpu, wl.config2(), num_splits=splits, hints=hints)


def test_config2_shape_at_batch_32(gpu):
    """The benchmark's saturating-batch extra (config 2's shape, 32 sequences): every output compared."""
    check_full(gpu, wl.config2(32), hints=True)


@pytest.mark.parametrize("hints", [True, False])
@pytest.mark.parametrize("B", [1, 4, 16, 64])
def test_config3_sweep(gpu, B, hints):
    check_full(gpu, wl.config3(B), hints=hints)


@pytest.mark.parametrize("hints", [True, False])
def test_config4_70b(gpu, hints):
    check_full(gpu, wl.config4(), hints=hints)


def test_config5_paged_reduced_lengths_full_compare(gpu):
    """Config 5's recipe at L_b in [1000, 3000]: every output compared."""
    check_full(gpu, wl.config5(l_lo=1000, l_hi=3000))


def test_config5_paged_full_size(gpu):
    """Config 5 at full size (L_b in [16384, 32768]) in the launch configuration the
    benchmark uses (automatic split count, length hint): every output compared with the oracle."""
    import torch
    w = wl.config5()
    say(f"[case] cfg5 full L={list(w.L)}")
    dw = gpu.to_device(w)
    lens = np.ascontiguousarray(w.L, dtype=np.int32)
    mask, out, lse = gpu.run_path(dw, sum_L=int(lens.sum()), L_host=lens)   # the benchmark passes the host's lengths too
    torch.cuda.synchronize()
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), orc.ancestor_mask(w.parent, w.cu_T))
    ro, rl = orc.tree_verify_attn(w)
    o = out.cpu().numpy().astype(np.float64)
    l = lse.cpu().numpy().astype(np.float64)
    assert np.isfinite(o).all() and np.isfinite(l).all()
    eo, el = np.abs(o - ro).max(), np.abs(l - rl).max()
    say(f"        all {o.shape[0] * o.shape[1]} rows: max|dO|={eo:.3e} max|dLSE|={el:.3e}")
    assert eo <= TOL_O and el <= TOL_LSE
    # property that holds at any size: constant V gives that constant back for every row
    v0 = wl.f32_to_bf16_bits(np.linspace(-1, 1, 128, dtype=np.float32))
    dw.v_cache[:] = torch.from_numpy(v0.view(np.int16)).to(dw.v_cache.device)
    dw.v_tree[:] = torch.from_numpy(v0.view(np.int16)).to(dw.v_tree.device)
    out2, _ = gpu.attention(dw, mask)
    torch.cuda.synchronize()
    dev = (out2.cpu().numpy() - wl.bf16_bits_to_f32(v0)[None, None, :])
    assert np.abs(dev).max() <= TOL_O


# ------------------------------------------------------------------ edge cases and sweeps
@pytest.mark.parametrize("L", [0, 1, 15, 16, 17, 63, 64, 65, 127, 128, 129, 200])
def test_cache_length_edges(gpu, L):
    check_full(gpu, wl.random_workload(100 + L, 2, 8, 2, 128, [L, max(0, L - 1)], [7, 12]), label=f"L={L}")


@pytest.mark.parametrize("T", [1, 2, 8, 9, 16, 31, 32, 33, 60, 64, 65, 72, 100, 128])
def test_tree_size_edges(gpu, T):
    """T = 72 is the paper's total_token; T > 64 uses two mask words."""
    check_full(gpu, wl.random_workload(200 + T, 1, 4, 2, 128, [75], [T], max_depth=13), label=f"T={T}")


@pytest.mark.parametrize("Hq,Hkv", [(4, 4), (8, 4), (8, 2), (8, 1), (16, 1), (6, 2), (12, 4), (10, 2), (14, 2), (7, 1)])
@pytest.mark.parametrize("D", [64, 128])
def test_gqa_groups_and_head_dims(gpu, Hq, Hkv, D):
    check_full(gpu, wl.random_workload(300 + Hq + Hkv + D, 2, Hq, Hkv, D, [150, 33], [20, 11]),
               label=f"Hq={Hq} Hkv={Hkv} D={D}")


@pytest.mark.parametrize("splits", [1, 2, 3, 5, 8, 100])
def test_split_counts_ragged(gpu, splits):
    """A race or a wrong split boundary shows as split-dependent output."""
    w = wl.random_workload(400, 4, 8, 2, 128, [700, 64, 0, 333], [24, 5, 9, 40])
    check_full(gpu, w, num_splits=splits, label=f"splits={splits}")


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5])
def test_every_workgroup_shape(gpu, variant):
    """Every workgroup shape of the kernel (tva_shape, named through tva_args.plan_shape) on inputs the
    planner would give to another one: dense with several splits and ragged tails, paged, and head
    dimension 64, all against the oracle."""
    check_full(gpu, wl.random_workload(700 + variant, 3, 8, 2, 128, [900, 130, 0], [70, 33, 8], max_depth=10),
               num_splits=3, label=f"shape {variant} dense", plan_shape=variant)
    check_full(gpu, wl.random_workload(720 + variant, 2, 8, 2, 128, [517, 64], [40, 64], page_size=16),
               label=f"shape {variant} paged", plan_shape=variant)
    check_full(gpu, wl.random_workload(740 + variant, 2, 8, 4, 64, [300, 77], [60, 9]),
               num_splits=2, label=f"shape {variant} D=64", plan_shape=variant)
    # and with the ancestor sets derived in the kernel: bit-identical to passing the masks
    import torch
    dw = gpu.to_device(wl.random_workload(760 + variant, 3, 8, 2, 128, [400, 70, 0], [72, 30, 5], max_depth=12))
    a = gpu.attention(dw, gpu.build_mask(dw), num_splits=2, plan_shape=variant)
    b = gpu.attention(dw, None, num_splits=2, plan_shape=variant)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


@pytest.mark.parametrize("B,L,T,page,rows,splits", [
    (8, 2048, 60, 0, 128, 2), (16, 2048, 60, 0, 128, 1), (20, 1024, 60, 0, 256, 1), (4, 8192, 60, 0, 256, 8),
    (4, 4096, 60, 0, 64, 4), (32, 1024, 16, 0, 64, 1), (8, 4096, 32, 0, 256, 4),
    (8, 2048, 60, 16, 128, 2), (20, 1024, 60, 16, 256, 1), (4, 4096, 60, 16, 64, 4),
])
def test_every_band_of_the_launch_planner(gpu, B, L, T, page, rows, splits):
    """Batch / length shapes that land in each band of the launch planner (workgroup rows and split count
    asserted), with ragged lengths and tree sizes below the maxima, planner left to itself."""
    from paper_2510_26577_amd import binding
    rng = np.random.Generator(np.random.PCG64(B * 131 + L + T))
    Ls = rng.integers(L // 2, L + 1, B)
    Ts = rng.integers(max(1, T - 8), T + 1, B)
    Ls[int(rng.integers(0, B))], Ts[int(rng.integers(0, B))] = L, T
    w = wl.random_workload(900 + B + L + T, B, 32, 8, 128, Ls, Ts, max_depth=8, page_size=page)
    a = binding.TvaArgs()
    a.B, a.Hq, a.Hkv, a.D, a.sum_T, a.max_T, a.mask_words, a.max_L, a.scale = B, 32, 8, 128, w.sum_T, T, 1, L, w.scale
    assert (binding.plan_workgroup_rows(a), binding.plan_splits(a)) == (rows, splits)
    check_full(gpu, w, label=f"planner band rows={rows} splits={splits} page={page}")


@pytest.mark.parametrize("page", [0, 16])
def test_length_hint_changes_the_plan_not_the_result(gpu, page):
    """Long ragged caches with their sum passed as the planning hint: shorter splits (asserted), same result."""
    import torch
    from paper_2510_26577_amd import binding
    L = [6000, 11900, 7100, 12000]
    w = wl.random_workload(950 + page, 4, 32, 8, 128, L, [48, 40, 48, 33], max_depth=7, page_size=page)
    a = binding.TvaArgs()
    a.B, a.Hq, a.Hkv, a.D, a.sum_T, a.max_T, a.mask_words, a.max_L, a.scale = 4, 32, 8, 128, w.sum_T, 48, 1, 12000, w.scale
    plain = binding.plan_chunk_keys(a)
    a.sum_L = sum(L)
    hinted = binding.plan_chunk_keys(a)
    say(f"[case] length hint page={page}: split {plain} -> {hinted} keys")
    assert hinted < plain
    dw = gpu.to_device(w)
    out, lse = gpu.attention(dw, None, sum_L=sum(L))
    out0, lse0 = gpu.attention(dw, None)
    torch.cuda.synchronize()
    ro, rl = orc.tree_verify_attn(w)
    for o, l in ((out, lse), (out0, lse0)):
        assert np.abs(o.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
        assert np.abs(l.cpu().numpy().astype(np.float64) - rl).max() <= TOL_LSE


@pytest.mark.parametrize("case", ["cfg2", "cfg3_B16", "cfg4", "cfg5", "ragged", "paged", "forest_T128", "D64"])
def test_masks_derived_in_kernel_equal_masks_passed(gpu, case):
    """Passing the parent arrays instead of ancestor masks gives the same ancestor sets, hence the same
    bits out (same arithmetic in the same order); the result is also checked against the oracle."""
    import torch
    w = {"cfg2": lambda: wl.config2(), "cfg3_B16": lambda: wl.config3(16),
         "cfg4": lambda: wl.config4(), "cfg5": lambda: wl.config5(),
         "ragged": lambda: wl.random_workload(800, 5, 8, 2, 128, [700, 64, 0, 333, 5], [24, 5, 0, 40, 1]),
         "paged": lambda: wl.random_workload(801, 3, 8, 2, 128, [517, 64, 130], [40, 64, 7], page_size=16),
         "forest_T128": lambda: wl.random_workload(802, 2, 4, 2, 128, [75, 0], [128, 100], max_depth=13),
         "D64": lambda: wl.random_workload(803, 2, 8, 4, 64, [300, 77], [60, 9])}[case]()
    if case == "forest_T128":                      # several roots in one tree
        w.parent[w.cu_T[0] + 5] = -1
        w.parent[w.cu_T[1] + 50] = -1
    say(f"[case] in-kernel masks: {case}")
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    for splits in (0, 1, 3):
        out_a, lse_a = gpu.attention(dw, mask, num_splits=splits)
        out_b, lse_b = gpu.attention(dw, None, num_splits=splits)
        torch.cuda.synchronize()
        assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b)
    ro, rl = orc.tree_verify_attn(w)
    assert np.abs(out_b.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
    assert np.abs(lse_b.cpu().numpy().astype(np.float64) - rl).max() <= TOL_LSE


@pytest.mark.parametrize("variant", [0, 1, 2, 3, 5])
@pytest.mark.parametrize("page_size", [0, 16])
def test_queries_are_the_last_nodes_of_each_tree(gpu, page_size, variant):
    """cu_Q: only the last Tq_b nodes of each tree are queries (the draft model's attention for the newest
    expansion layer); keys stay all T_b nodes.  Rows must equal the oracle's rows of those nodes."""
    import torch
    from paper_2510_26577_amd import binding
    w = wl.random_workload(1200 + page_size, 5, 8, 2, 128, [400, 70, 0, 33, 129], [72, 30, 5, 12, 128], max_depth=13,
                           page_size=page_size)
    Tq = np.array([12, 30, 1, 0, 60])                    # newest layer sizes (whole tree, one node, none, ...)
    cu_Q = np.concatenate([[0], np.cumsum(Tq)]).astype(np.int32)
    sel = np.concatenate([np.arange(w.cu_T[b + 1] - Tq[b], w.cu_T[b + 1]) for b in range(w.B)]).astype(np.int64)
    say(f"[case] query subset page_size={page_size} variant={variant} Tq={list(Tq)}")
    dw = gpu.to_device(w)
    q_sub = dw.q[torch.from_numpy(sel).to(dw.q.device)].contiguous()
    ro, rl = orc.tree_verify_attn(w)
    mask = gpu.build_mask(dw)
    for use_mask in (True, False):
        for splits in (0, 3):
            out, lse = binding.tree_verify_attn(
                q_sub, dw.k_tree, dw.v_tree, dw.k_cache, dw.v_cache, mask if use_mask else None, dw.cu_T, dw.L,
                max_T=w.max_T, max_L=w.max_L, scale=w.scale, cu_L=dw.cu_L, page_table=dw.page_table,
                page_size=w.page_size, num_splits=splits, parent=None if use_mask else dw.parent,
                cu_Q=torch.from_numpy(cu_Q).to(dw.q.device), max_Q=int(Tq.max()), plan_shape=variant)
            torch.cuda.synchronize()
            assert out.shape[0] == len(sel)
            eo = np.abs(out.cpu().numpy().astype(np.float64) - ro[sel]).max()
            el = np.abs(lse.cpu().numpy().astype(np.float64) - rl[sel]).max()
            assert eo <= TOL_O and el <= TOL_LSE


def test_empty_trees_in_batch_and_chain_and_star(gpu):
    rng = np.random.Generator(np.random.PCG64(500))
    trees = [wl.tree_chain(13), np.zeros(0, np.int32), wl.tree_star(30), wl.tree_chain(1)]
    w = wl.make_workload("shapes", 500, 4, 8, 4, 128, [90, 50, 260, 0], trees, rng=rng)
    check_full(gpu, w, num_splits=2)


def test_forest_with_several_roots(gpu):
    rng = np.random.Generator(np.random.PCG64(501))
    t = wl.tree_uniform(rng, 40, 6)
    t[[9, 21]] = -1
    w = wl.make_workload("forest", 501, 1, 4, 4, 64, [0], [t], rng=rng)
    check_full(gpu, w)


def test_paged_nan_tails_and_unused_pages(gpu):
    """Slots past L_b in the last page and unused pool pages hold NaN: never read."""
    w = wl.random_workload(502, 3, 8, 2, 128, [37, 64, 5], [9, 17, 3], page_size=16)
    used = np.zeros(w.k_cache.shape[:2], dtype=bool)
    for b in range(3):
        for t in range(int(w.L[b])):
            used[w.page_table[b, t // 16], t % 16] = True
    w.k_cache[~used] = 0x7FC0
    w.v_cache[~used] = 0x7FC0
    spare = int(np.flatnonzero(~used.any(axis=1))[0])   # an unused, all-NaN page
    w.page_table[w.page_table < 0] = spare              # entries past the last page: valid index, poisoned data
    check_full(gpu, w, num_splits=2)


def test_head_major_pool_strides(gpu):
    """The same paged cache stored head-major: [page, head, slot, d] via strides."""
    import torch
    w = wl.random_workload(503, 2, 8, 2, 128, [100, 47], [10, 6], page_size=16)
    ro, rl = orc.tree_verify_attn(w)
    dw = gpu.to_device(w)
    dw.k_cache = dw.k_cache.permute(0, 2, 1, 3).contiguous()   # [P, Hkv, 16, D]
    dw.v_cache = dw.v_cache.permute(0, 2, 1, 3).contiguous()
    mask = gpu.build_mask(dw)
    out, lse = gpu.attention(dw, mask, strides=(w.Hkv * 16 * w.D, w.D, 16 * w.D))
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - ro).max() <= TOL_O and np.abs(lse.cpu().numpy() - rl).max() <= TOL_LSE


def test_all_true_mask_is_full_attention(gpu):
    """Masking with all-true ancestor bits reproduces unmasked attention over L+T keys:
    compared with the oracle on a chain whose last node sees everything."""
    import torch
    rng = np.random.Generator(np.random.PCG64(504))
    T = 20
    w = wl.make_workload("full", 504, 1, 4, 2, 128, [77], [wl.tree_chain(T)], rng=rng)
    ro, rl = orc.tree_verify_attn(w)
    dw = gpu.to_device(w)
    mask = torch.full((T, 1), (1 << T) - 1, dtype=torch.int64, device="cuda:0")
    out, lse = gpu.attention(dw, mask)
    torch.cuda.synchronize()
    # only the last node's reference row is "all keys"; its query is row T-1
    assert np.abs(out.cpu().numpy()[T - 1] - ro[T - 1]).max() <= TOL_O
    assert np.abs(lse.cpu().numpy()[T - 1] - rl[T - 1]).max() <= TOL_LSE


def test_max_L_bound_larger_than_lengths(gpu):
    """max_L is only an upper bound: a loose bound changes the launch, not the result."""
    import torch
    w = wl.random_workload(505, 2, 8, 2, 128, [130, 20], [12, 12])
    ro, rl = orc.tree_verify_attn(w)
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    out, lse = gpu.attention(dw, mask, max_L=4096, num_splits=7)
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - ro).max() <= TOL_O and np.abs(lse.cpu().numpy() - rl).max() <= TOL_LSE


def test_ancestor_mask_many_trees_bit_exact(gpu):
    import torch
    rng = np.random.Generator(np.random.PCG64(506))
    trees = [wl.tree_uniform(rng, int(t), int(d)) for t, d in
             zip(rng.integers(1, 129, size=300), rng.integers(1, 14, size=300))]
    trees += [wl.tree_chain(128), wl.tree_star(128), wl.tree_chain(64), wl.tree_chain(65)]
    cu_T = np.zeros(len(trees) + 1, np.int32)
    cu_T[1:] = np.cumsum([len(t) for t in trees])
    parent = np.concatenate(trees).astype(np.int32)
    from paper_2510_26577_amd import binding
    err = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    m = binding.build_ancestor_mask(torch.from_numpy(parent).cuda(), torch.from_numpy(cu_T).cuda(), 128, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    assert np.array_equal(m.cpu().numpy().view(np.uint64), orc.ancestor_mask(parent, cu_T, words=2))


def test_ancestor_mask_reports_malformed_tree(gpu):
    import torch
    from paper_2510_26577_amd import binding
    parent = np.array([-1, 0, 1, -1, 2, 0, -1, 0, 5], np.int32)  # tree 1 (nodes 3..5): node 4 -> parent 2 >= 1
    cu_T = np.array([0, 3, 6, 9], np.int32)
    parent[7] = 1                                                 # tree 2: node 1 -> parent 1 (self)
    err = torch.zeros(1, dtype=torch.int32, device="cuda:0")
    binding.build_ancestor_mask(torch.from_numpy(parent).cuda(), torch.from_numpy(cu_T).cuda(), 3, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 4 + 1                               # smallest offending global index, plus one
    with pytest.raises(ValueError):
        orc.ancestor_mask(parent, cu_T)


def test_merge_splits_entry_point(gpu):
    import torch
    from paper_2510_26577_amd import binding
    rng = np.random.Generator(np.random.PCG64(507))
    for D in (64, 128):
        S, n = 5, 37
        po = rng.standard_normal((S, n, D)).astype(np.float32)
        pl = (rng.standard_normal((S, n)) * 3).astype(np.float32)
        pl[2, :] = -np.inf            # an empty partial
        pl[:, 5] = -np.inf            # a row with no key at all
        ro, rl = orc.merge_splits(po, pl)
        out, lse = binding.merge_splits(torch.from_numpy(po).cuda(), torch.from_numpy(pl).cuda())
        torch.cuda.synchronize()
        o, l = out.cpu().numpy(), lse.cpu().numpy()
        assert np.all(o[5] == 0) and l[5] == -np.inf
        keep = np.arange(n) != 5
        assert np.abs(o[keep] - ro[keep]).max() <= 1e-5 and np.abs(l[keep] - rl[keep]).max() <= 1e-5


def test_repeated_calls_are_deterministic(gpu):
    import torch
    w = wl.config3(4)
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    a, la = gpu.attention(dw, mask, num_splits=4)
    b, lb = gpu.attention(dw, mask, num_splits=4)
    torch.cuda.synchronize()
    assert torch.equal(a, b) and torch.equal(la, lb)


@pytest.mark.parametrize("B,T", [(64, 8), (48, 3), (33, 16), (64, 1)])
def test_host_lengths_hint_changes_nothing_but_the_placement(gpu, B, T):
    """tva_args.L_host only decides which workgroup slot takes which sequence (ragged batches of 33 .. 64 sequences
    with 8 KV heads and up to 64 rows per KV head): the true lengths, reversed ones and nonsense all give bit for bit
    what no hint gives, and that agrees with the oracle."""
    import torch
    rng = np.random.Generator(np.random.PCG64(500 + B + T))
    L = rng.integers(0, 700, size=B)
    L[:3] = [0, 699, 1]
    w = wl.random_workload(900 + B, B, 32, 8, 128, L, T, max_depth=6)
    say(f"[case] length hint B={B} T={T}")
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    base, lbase = gpu.attention(dw, mask)
    torch.cuda.synchronize()
    ro, rl = orc.tree_verify_attn(w)
    assert np.abs(base.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
    assert np.abs(lbase.cpu().numpy().astype(np.float64) - rl).max() <= TOL_LSE
    for hint in (w.L, w.L[::-1], np.full(B, 7), rng.integers(-5, 10 ** 9, size=B)):
        o, l = gpu.attention(dw, mask, L_host=np.ascontiguousarray(hint, dtype=np.int32))
        torch.cuda.synchronize()
        assert torch.equal(o, base) and torch.equal(l, lbase)


@pytest.mark.parametrize("L,T", [([5000, 2300, 7900], 16), ([9000, 20000], 64), ([1500, 1100, 6000, 3000, 200], 40)])
def test_host_lengths_hint_in_split_launches_matches_oracle(gpu, L, T):
    """With KV splits the host's lengths shorten the splits (the planner counts the non-empty ones): the outputs
    agree with the oracle with the hint, without it, and with lengths that are not the batch's."""
    import torch
    from paper_2510_26577_amd import binding
    B = len(L)
    w = wl.random_workload(700 + B + T, B, 32, 8, 128, np.array(L), T, max_depth=8)
    say(f"[case] length hint with splits L={L} T={T}")
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    ro, rl = orc.tree_verify_attn(w)
    hints = (None, np.ascontiguousarray(w.L, dtype=np.int32), np.full(B, 1234, dtype=np.int32))
    for hint in hints:
        o, l = gpu.attention(dw, mask, L_host=hint, sum_L=0 if hint is None else int(w.L.sum()))
        torch.cuda.synchronize()
        assert np.abs(o.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
        assert np.abs(l.cpu().numpy().astype(np.float64) - rl).max() <= TOL_LSE
    a = binding.TvaArgs()
    a.B, a.Hq, a.Hkv, a.D, a.sum_T, a.max_T, a.mask_words, a.max_L = B, 32, 8, 128, B * T, T, (T + 63) // 64, max(L)
    lens = np.ascontiguousarray(w.L, dtype=np.int32)
    plain = binding.plan_chunk_keys(a)
    a.L_host = lens.ctypes.data
    assert binding.plan_chunk_keys(a) <= plain


@pytest.mark.parametrize("splits", [2, 3, 7])
def test_splits_entry_point_partials_match_oracle_key_ranges(gpu, splits):
    """tva_tree_verify_attn_splits leaves per-split partials that equal the oracle restricted to
    each split's keys; merging them with tva_merge_splits gives the full result."""
    import torch
    from paper_2510_26577_amd import binding
    w = wl.random_workload(600 + splits, 2, 8, 2, 128, [700, 300], [24, 9])
    dw = gpu.to_device(w)
    mask = gpu.build_mask(dw)
    out = torch.zeros((w.sum_T, w.Hq, w.D), dtype=torch.float32, device="cuda:0")
    lse = torch.zeros((w.sum_T, w.Hq), dtype=torch.float32, device="cuda:0")
    args = binding.make_args(q=dw.q, k_tree=dw.k_tree, v_tree=dw.v_tree, k_cache=dw.k_cache, v_cache=dw.v_cache,
                             anc_mask=mask, cu_T=dw.cu_T, L=dw.L, max_T=w.max_T, max_L=w.max_L, scale=w.scale,
                             cu_L=dw.cu_L, num_splits=splits, out=out, lse=lse)
    S, ck = binding.plan_splits(args), binding.plan_chunk_keys(args)
    assert S >= 2
    ws = torch.empty(binding.workspace_bytes(args) // 4, dtype=torch.float32, device="cuda:0")
    args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel() * 4
    binding.tree_verify_attn_splits_raw(args)
    torch.cuda.synchronize()
    n = w.sum_T * w.Hq
    po = ws[: S * n * w.D].view(S, n, w.D)
    pl = ws[S * n * w.D: S * n * (w.D + 1)].view(S, n)
    for b in range(w.B):
        Lb, r0, r1 = int(w.L[b]), int(w.cu_T[b]) * w.Hq, int(w.cu_T[b + 1]) * w.Hq
        nc = max(1, -(-Lb // ck))
        for s in range(S):
            got_l = pl[s, r0:r1].cpu().numpy()
            if s >= nc:
                assert np.all(np.isneginf(got_l))
                continue
            hi = Lb + int(w.T[b]) if s == nc - 1 else (s + 1) * ck
            rows = [(b, i, h) for i in range(int(w.T[b])) for h in range(w.Hq)]
            ro, rl = orc.tree_verify_attn(w, rows=rows, key_range=(s * ck, hi))
            assert np.abs(got_l - rl).max() <= TOL_LSE
            assert np.abs(po[s, r0:r1].cpu().numpy() - ro).max() <= TOL_O
    binding.merge_splits(po, pl, out=out.view(n, w.D), lse=lse.view(n))
    torch.cuda.synchronize()
    fo, fl = orc.tree_verify_attn(w)
    assert np.abs(out.cpu().numpy() - fo).max() <= TOL_O and np.abs(lse.cpu().numpy() - fl).max() <= TOL_LSE


@pytest.mark.parametrize("seed", list(range(24)))
def test_seeded_random_shapes(gpu, seed):
    """Valid shapes drawn at random (fixed seeds): head counts and group sizes, head dimension, ragged cache and
    tree sizes including empty ones, dense or paged with odd page sizes, automatic or forced splits, masks
    passed or derived in the kernel -- each against the oracle."""
    import torch
    rng = np.random.Generator(np.random.PCG64(7000 + seed))
    B = int(rng.integers(1, 7))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 4, 7, 8]))
    D = int(rng.choice([64, 128]))
    L = rng.integers(0, int(rng.choice([40, 300, 900])) + 1, B)
    T = rng.integers(0, int(rng.choice([8, 40, 128])) + 1, B)
    T[int(rng.integers(0, B))] = max(1, int(T.max()))
    page = int(rng.choice([0, 0, 1, 5, 16, 64]))
    splits = int(rng.choice([0, 0, 1, 2, 5]))
    w = wl.random_workload(7100 + seed, B, Hkv * G, Hkv, D, L, T, max_depth=int(rng.integers(1, 14)), page_size=page)
    say(f"[case] random seed={seed} B={B} Hkv={Hkv} G={G} D={D} L={list(L)} T={list(T)} page={page} splits={splits}")
    check_full(gpu, w, num_splits=splits, label=f"random {seed}", hints=seed % 2 == 1)
    dw = gpu.to_device(w)
    out, lse = gpu.attention(dw, None, num_splits=splits, sum_L=int(L.sum()))
    torch.cuda.synchronize()
    ro, rl = orc.tree_verify_attn(w)
    if ro.size:
        assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= TOL_O
        fin = np.isfinite(rl)
        assert np.array_equal(np.isfinite(lse.cpu().numpy()), fin)
        assert np.abs(lse.cpu().numpy().astype(np.float64)[fin] - rl[fin]).max() <= TOL_LSE if fin.any() else True
