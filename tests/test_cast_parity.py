"""Native tree-size selection (libtva host entry points, through the C ABI) against the CPU oracle
on the same seeded inputs.  Integer results must agree exactly; the floating-point intermediates
(utilities, costs, buffer averages) to a few ulps -- the two sides sum in different orders, and a
kept count can only differ where a chord sits within that rounding of the threshold, which the
random cases check for and the exact (dyadic) cases exclude by construction.  Host logic: no GPU."""
import os

import numpy as np
import pytest

from oracle import cast_oracle as co
from paper_2510_26577_amd import binding, cast


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(binding.LIB_PATH):
        binding.build_library()
    return binding.load_library()


def tables(rng, M, N, draft_scale=0.1):
    """Cost tables shaped like measured ones: increasing in context and in tokens, mildly convex."""
    n = np.arange(1, N + 1)
    S_T = np.stack([(50.0 + 5.0 * r) + (0.4 + 0.05 * r) * n + 0.002 * n * n + rng.uniform(0, 0.01, N).cumsum()
                    for r in range(1, M + 1)])
    S_D = draft_scale * np.stack([(20.0 + 2.0 * r) + (0.3 + 0.02 * r) * n + rng.uniform(0, 0.01, N).cumsum()
                                  for r in range(1, M + 1)])
    return S_D, S_T


def sorted_scores(rng, B, N):
    return (-np.sort(-rng.random((B, N)) ** 2, axis=1)).astype(np.float32)


def chord_margin(u, c, C):
    u, c = np.asarray(u, float), np.asarray(c, float)
    j, i = np.triu_indices(len(u), 1)[::-1]
    ch = (u[j] - u[i]) / (c[j] - c[i])
    return np.min(np.abs(ch - C)) if len(ch) else np.inf


def test_select_context_matches_oracle():
    for L, M in [(1, 1), (64, 4), (256, 8), (100, 3)]:
        for c in list(range(0, 5 * L * M // 4 + 3, max(1, L // 7))) + [10 ** 6]:
            assert cast.select_context(c, L, M) == co.select_context(c, L, M)
    with pytest.raises(binding.TvaError):
        cast.select_context(-1, 64, 4)


def test_algorithm_1_random_and_exact_ties():
    rng = np.random.Generator(np.random.PCG64(11))
    for _ in range(300):
        n = int(rng.integers(1, 73))
        u = np.cumsum(rng.normal(0.3, 0.5, n))          # not monotone, not concave
        c = np.cumsum(rng.uniform(0.05, 1.0, n))
        C = float(rng.uniform(0.01, 2.0))
        assert cast.select_max_valid_index(u, c, C) == co.select_max_valid_index(u, c, C)
    # exact ties: dyadic values, chords equal to the threshold must keep their mark on both sides
    for _ in range(100):
        n = int(rng.integers(2, 20))
        u = np.cumsum(rng.integers(-2, 6, n)).astype(float)
        c = np.cumsum(rng.integers(1, 4, n)).astype(float)
        for C in (0.25, 0.5, 1.0, 2.0):
            assert cast.select_max_valid_index(u, c, C) == co.select_max_valid_index(u, c, C)
    assert cast.select_max_valid_index([1, 2, 2.1, 4], [1, 2, 3, 4], 0.5) == 4     # the hand-worked case
    with pytest.raises(binding.TvaError):
        cast.select_max_valid_index([1, 2, 3], [1, 1, 2], 0.5)                      # c not strictly increasing


def test_utility_cost_and_breadth_pruning():
    rng = np.random.Generator(np.random.PCG64(12))
    checked = 0
    for _ in range(120):
        B, N, M, L = int(rng.integers(1, 65)), int(rng.integers(1, 33)), int(rng.integers(1, 9)), 128
        S_D, S_T = tables(rng, M, 72)
        s = sorted_scores(rng, B, N)
        ctx = int(rng.integers(0, (M + 2) * L))
        u_ref, c_ref = co.layer_utility(s), co.layer_cost(S_D, S_T, ctx, L, M, N)
        assert np.allclose(cast.layer_utility(s), u_ref, rtol=1e-13, atol=0)
        assert np.array_equal(cast.layer_cost(S_D, S_T, ctx, L, N), np.array(c_ref))
        C1 = float(10.0 ** rng.uniform(0.0, 3.7))       # from keep-everything to keep-one
        if chord_margin(u_ref, c_ref, C1) < 1e-9:
            continue
        n_ref, u_at, c_at = co.breadth_prune(s, S_D, S_T, ctx, L, M, C1)
        n_i, u_n, c_n = cast.breadth_prune(s, S_D, S_T, ctx, L, C1)
        assert n_i == n_ref and u_n == pytest.approx(u_at, rel=1e-13) and c_n == c_at
        checked += 1
    assert checked > 100


def test_theorem_through_the_native_path():
    """Linear cost and the threshold of the paper's theorem: exactly K nodes are kept."""
    rng = np.random.Generator(np.random.PCG64(13))
    for B, N, K in [(1, 8, 3), (4, 16, 5), (16, 10, 10), (64, 12, 1)]:
        s = sorted_scores(rng, B, N)
        lam, delta = 0.37, 1.9
        S_D = np.array([[lam * j + delta for j in range(1, N + 1)]])
        S_T = np.ones((1, N))
        C1 = float(s[:, K - 1].astype(np.float64).sum() / (B * lam)) * (1 - 1e-9)
        assert cast.breadth_prune(s, S_D, S_T, ctx=0, L=64, C1=C1)[0] == K


def test_depth_buffers_follow_the_oracle():
    rng = np.random.Generator(np.random.PCG64(14))
    for R in (1, 2, 5):
        nat, ref = cast.DepthPruner(max_layers=6, R=R, C2=0.8), co.DepthPruner(R=R, C2=0.8)
        for _ in range(60):
            layer = int(rng.integers(1, 7))
            u1, u0, cc = float(rng.uniform(0.1, 3)), float(rng.uniform(0.1, 3)), float(rng.uniform(0.1, 3))
            assert nat.alpha(layer) == pytest.approx(ref.alpha(layer), rel=1e-14)
            if abs(ref.alpha(layer) * u0 / cc - 0.8) > 1e-9:
                assert nat.should_expand(layer, u0, cc) == ref.should_expand(layer, u0, cc)
            assert nat.update(layer, u1, u0) == ref.update(layer, u1, u0)
    assert np.isnan(cast.DepthPruner(3, 2, 1.0).alpha(4))


def test_expansion_plan_matches_oracle():
    rng = np.random.Generator(np.random.PCG64(15))
    L, M = 64, 6
    S_D, S_T = tables(rng, M, 72)
    agree = 0
    nat, ref = cast.DepthPruner(max_layers=8, R=4, C2=12.0), co.DepthPruner(R=4, C2=12.0)
    for step in range(40):                       # the buffers persist from one decode step to the next
        B = 4
        decay = rng.uniform(0.3, 0.95)
        layers = [sorted_scores(rng, B, int(rng.integers(2, 13))) * np.float32(decay ** d) for d in range(8)]
        C1 = float(10.0 ** rng.uniform(1.0, 3.3))
        kept_ref = co.expansion_plan(layers, S_D, S_T, n0=17, L=L, M=M, C1=C1, pruner=ref)
        kept = cast.expansion_plan(layers, S_D, S_T, n0=17, L=L, C1=C1, pruner=nat)
        assert kept == kept_ref
        agree += 1
        for layer in range(1, 9):
            assert nat.alpha(layer) == pytest.approx(ref.alpha(layer), rel=1e-12)
    assert agree == 40


def test_expansion_plan_hand_worked_case_through_the_native_path():
    """The hand-worked two-step case of tests/cast_cases.py (expected values from paper arithmetic,
    not from the oracle): kept counts and every buffer average, exactly."""
    import cast_cases as cc
    pr = cast.DepthPruner(max_layers=4, R=cc.R, C2=cc.C2)
    assert cast.expansion_plan(cc.STEP1, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, C1=cc.C1, pruner=pr) == cc.KEPT1
    for layer, a in cc.ALPHA_AFTER_1.items():
        assert pr.alpha(layer) == pytest.approx(a, rel=1e-7)   # the native scores are float32
    assert cast.expansion_plan(cc.STEP2, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, C1=cc.C1, pruner=pr) == cc.KEPT2
    for layer, a in cc.ALPHA_AFTER_2.items():
        assert pr.alpha(layer) == pytest.approx(a, rel=1e-7)
    fresh = cast.DepthPruner(max_layers=4, R=cc.R, C2=cc.C2)
    assert cast.expansion_plan(cc.STEP2, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, C1=cc.C1, pruner=fresh) == [3, 2, 2]


def test_rerank_count_and_subtree_selection():
    rng = np.random.Generator(np.random.PCG64(16))
    L, M = 128, 8
    S_D, S_T = tables(rng, M, 72)
    for _ in range(60):
        B, N_tot, m = int(rng.integers(1, 33)), int(rng.integers(1, 100)), int(rng.integers(1, 73))
        tree = (rng.random((B, N_tot)) ** 3).astype(np.float32)
        C3, n0 = float(rng.uniform(0.5, 40.0)), int(rng.integers(0, 2000))
        assert cast.rerank_count(tree, S_T, n0, L, m, C3) == co.rerank_count(tree, S_T, n0, L, M, m, C3)
    for n in (1, 2, 17, 60, 128):
        parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, n)], np.int32)
        score = np.ones(n, np.float32)
        for i in range(1, n):
            score[i] = score[parent[i]] * np.float32(rng.choice([0.25, 0.5, 0.5, 0.75, 1.0]))   # ties on purpose
        for keep in sorted({1, max(1, n // 3), n}):
            old, newp = cast.select_subtree(score, parent, keep)
            old_ref, newp_ref = co.select_subtree(score, parent, keep)
            assert list(old) == old_ref and list(newp) == newp_ref
    with pytest.raises(binding.TvaError):
        cast.select_subtree([1.0, 0.1, 0.9], [-1, 0, 1], 2)


def test_selected_subtree_feeds_the_mask_oracle():
    """The relabelled parent array is a valid input of the verification attention: topological, one root."""
    from oracle import tva_oracle as orc
    rng = np.random.Generator(np.random.PCG64(17))
    n = 90
    parent = np.array([-1] + [int(rng.integers(max(0, i - 9), i)) for i in range(1, n)], np.int32)
    score = np.ones(n, np.float32)
    for i in range(1, n):
        score[i] = score[parent[i]] * np.float32(rng.uniform(0.2, 0.99))
    old, newp = cast.select_subtree(score, parent, 60)
    mask = orc.ancestor_mask(newp.astype(np.int32), np.array([0, 60], np.int32))
    full = orc.ancestor_mask(parent, np.array([0, n], np.int32), words=2)
    for k, o in enumerate(old):     # ancestors of a kept node in the subtree = its ancestors in the full tree
        anc_full = {j for j in range(n) if (int(full[o, j // 64]) >> (j % 64)) & 1}
        anc_sub = {int(old[j]) for j in range(60) if (int(mask[k, 0]) >> j) & 1}
        assert anc_sub == anc_full
