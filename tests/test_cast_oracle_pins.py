"""Pins of the CAST host-logic oracle (oracle/cast_oracle.py) against what the paper and the
mathematics fix: the paper's theorem (linear cost => the EAGLE top-K rule), closed forms for
concave utilities, limits in the threshold, a hand-worked non-concave case, and the table-row
selector's grid.  CPU only."""
import itertools

import numpy as np
import pytest

from oracle import cast_oracle as co


def test_theorem_linear_cost_returns_top_k():
    """Method, Theorem: with c_j = lambda*j + delta and C1 = sum_j v_i^(j)(K) / (B*lambda) the selection
    keeps exactly K nodes (scores strictly decreasing so that no tie extends the kept set)."""
    rng = np.random.Generator(np.random.PCG64(1))
    for B, N, K in itertools.product([1, 3, 8], [4, 10, 25], [1, 2, 4]):
        scores = -np.sort(-rng.random((B, N)), axis=1)
        lam, delta = float(rng.uniform(0.01, 2.0)), float(rng.uniform(0.0, 3.0))
        u = co.layer_utility(scores)
        c = [lam * j + delta for j in range(1, N + 1)]
        C1 = scores[:, K - 1].sum() / (B * lam)
        # guard against rounding on the boundary chord itself
        assert co.select_max_valid_index(u, c, C1 * (1 - 1e-12)) == K


def test_concave_utility_closed_form():
    """For a concave u(c) the smallest chord ending at j is the last segment, so the result is the
    last index whose own marginal utility reaches C."""
    rng = np.random.Generator(np.random.PCG64(2))
    for _ in range(50):
        n = int(rng.integers(2, 30))
        steps_c = rng.uniform(0.1, 1.0, n)
        slopes = -np.sort(-rng.uniform(0.0, 5.0, n))  # decreasing marginal utility
        c = np.cumsum(steps_c)
        u = np.cumsum(slopes * steps_c)
        C = float(rng.uniform(0.0, 5.0))
        expect = 1
        for j in range(1, n):
            if slopes[j] >= C:
                expect = j + 1
        # chords are recomputed from u and c: stay clear of thresholds within rounding of a slope
        if np.min(np.abs(slopes - C)) < 1e-9:
            continue
        assert co.select_max_valid_index(u, c, C) == expect


def test_threshold_limits_and_monotonicity():
    rng = np.random.Generator(np.random.PCG64(3))
    u = np.cumsum(rng.uniform(0.1, 1.0, 12))
    c = np.cumsum(rng.uniform(0.1, 1.0, 12))
    assert co.select_max_valid_index(u, c, 1e-9) == 12      # every chord of an increasing u is positive
    assert co.select_max_valid_index(u, c, 1e9) == 1        # index 1 is never unmarked
    prev = 12
    for C in np.linspace(0.0, 12.0, 60):
        k = co.select_max_valid_index(u, c, float(C))
        assert k <= prev
        prev = k


def test_hand_worked_non_concave_case():
    """u = (1, 2, 2.1, 4), c = (1, 2, 3, 4), C = 0.5.  Chords: 1->2: 1, 1->3: 0.55, 2->3: 0.1 (< C,
    index 3 unmarked), 1->4: 1, 2->4: 1, 3->4: 1.9.  Index 4 keeps its mark: the flat spot at 3 does
    not stop the selection, which is what the double loop buys over a first-failure rule."""
    assert co.select_max_valid_index([1, 2, 2.1, 4], [1, 2, 3, 4], 0.5) == 4
    # a threshold just above 1 also fails the chords 1->2, 1->4 and 2->4 (all equal to 1): only index 1 is left
    assert co.select_max_valid_index([1, 2, 2.1, 4], [1, 2, 3, 4], 1.0 + 1e-9) == 1
    assert co.select_max_valid_index([1, 2, 2.1, 4], [1, 2, 3, 4], 1.0) == 4


def test_select_context_grid():
    L, M = 256, 8
    assert co.select_context(0, L, M) == L
    assert co.select_context(L - 1, L, M) == L
    assert co.select_context(L, L, M) == 2 * L
    assert co.select_context(3 * L + 17, L, M) == 4 * L
    assert co.select_context((M - 1) * L, L, M) == M * L
    assert co.select_context(100 * L, L, M) == M * L          # clamped to the last row
    for c in range(0, 10 * L, 37):
        s = co.select_context(c, L, M)
        assert s % L == 0 and L <= s <= M * L and (s > c or s == M * L)


def test_utility_is_batch_mean_of_prefix_sums():
    rng = np.random.Generator(np.random.PCG64(4))
    scores = -np.sort(-rng.random((5, 9)), axis=1)
    u = np.array(co.layer_utility(scores))
    assert np.allclose(u, np.cumsum(scores, axis=1).mean(axis=0), rtol=1e-13)
    one = co.layer_utility(scores[:1])
    assert np.allclose(one, np.cumsum(scores[0]))
    assert np.allclose(co.layer_utility(np.repeat(scores[:1], 4, axis=0)), one)


def test_cost_is_draft_row_over_target_first_entry():
    L, M, N = 128, 4, 6
    S_D = [[10.0 * r + n for n in range(1, N + 1)] for r in range(1, M + 1)]
    S_T = [[100.0 * r + 3 * n for n in range(1, N + 1)] for r in range(1, M + 1)]
    c = co.layer_cost(S_D, S_T, ctx=130, L=L, M=M, n_candidates=4)     # select(130) = 2L -> row 2
    assert c == [(20.0 + k) / 203.0 for k in range(1, 5)]


def test_depth_pruner_fifo_and_start_value():
    p = co.DepthPruner(R=3, C2=0.5)
    assert p.alpha(1) == 1.0                                           # buffers start as {1}
    assert p.should_expand(1, u_ni=2.0, c_ni=4.0)                      # 1 * 2/4 >= 0.5
    assert not p.should_expand(1, u_ni=1.9, c_ni=4.0)
    for phi in (0.5, 0.25, 0.75):
        p.update(1, phi, 1.0)
    assert list(p.A[1]) == [0.5, 0.25, 0.75]                           # the initial 1 was pushed out
    assert p.alpha(1) == pytest.approx(0.5)
    p.update(1, 0.1, 1.0)
    assert list(p.A[1]) == [0.25, 0.75, 0.1]
    assert p.alpha(2) == 1.0                                           # one buffer per layer


def test_rerank_count_with_linear_target_cost():
    """Linear target cost: c_k = (a + b*k)/(a + b), so chords are v(k)*(a+b)/b for the concave prefix sums
    and the count is the number of rank-averaged scores that reach C3*b/(a+b)."""
    rng = np.random.Generator(np.random.PCG64(5))
    B, Ntot, L, M = 4, 40, 64, 6
    tree = rng.random((B, Ntot))
    a, b = 50.0, 2.0
    S_T = [[a + b * n for n in range(1, 73)] for _ in range(M)]
    v = np.sort(tree, axis=1)[:, ::-1].mean(axis=0)
    for C3 in (1.0, 5.0, 10.0, 20.0):
        thr = C3 * b / (a + b)
        expect = max(1, int((v[:30] >= thr).sum()))
        if np.min(np.abs(v[:30] - thr)) < 1e-9:
            continue
        assert co.rerank_count(tree, S_T, n0=100, L=L, M=M, m=30, C3=C3) == expect


def test_select_subtree_keeps_a_parent_closed_top_set():
    rng = np.random.Generator(np.random.PCG64(6))
    n = 60
    parent = [-1] + [int(rng.integers(0, i)) for i in range(1, n)]
    score = [1.0] * n
    for i in range(1, n):
        score[i] = score[parent[i]] * float(rng.uniform(0.05, 0.95))
    for keep in (1, 7, 30, 60):
        old, newp = co.select_subtree(score, parent, keep)
        assert len(old) == keep and old == sorted(old) and old[0] == 0
        thr = sorted(score, reverse=True)[keep - 1]
        assert all(score[i] >= thr for i in old)
        for k, o in enumerate(old):
            assert (newp[k] == -1 and parent[o] == -1) or old[newp[k]] == parent[o]
            assert newp[k] < k
    with pytest.raises(ValueError):
        co.select_subtree([1.0, 0.1, 0.9], [-1, 0, 1], 2)              # child outscoring its parent


def test_expansion_plan_stops_when_gain_drops():
    L, M, N = 64, 4, 8
    S_D = [[1.0 + 0.1 * n for n in range(1, N + 1)] for _ in range(M)]
    S_T = [[10.0 + 0.2 * n for n in range(1, N + 1)] for _ in range(M)]
    strong = [[0.9, 0.5, 0.3, 0.1]] * 2
    weak = [[0.02, 0.01, 0.005, 0.001]] * 2
    kept = co.expansion_plan([strong, strong, weak, strong], S_D, S_T, n0=0, L=L, M=M, C1=1.0,
                             pruner=co.DepthPruner(R=4, C2=1.0))
    # layer 3's utility at its kept size is far below C2 * cost: layer 4 is never generated
    assert len(kept) == 3 and all(1 <= k <= 4 for k in kept)


def test_expansion_plan_hand_worked_three_layers_two_steps():
    """The context of Eq. 2 grows with the nodes kept so far (the table row changes from layer to
    layer), phi_i goes into the buffer of layer i (not i+1), buffers persist from one decode step to
    the next and drop their oldest value: all worked out by hand in tests/cast_cases.py."""
    import cast_cases as cc
    pr = co.DepthPruner(R=cc.R, C2=cc.C2)
    kept = co.expansion_plan(cc.STEP1, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, M=cc.M, C1=cc.C1, pruner=pr)
    assert kept == cc.KEPT1
    for layer, a in cc.ALPHA_AFTER_1.items():
        assert pr.alpha(layer) == pytest.approx(a, rel=1e-12)
    for layer, buf in cc.BUFFERS_AFTER_1.items():
        assert list(pr.A[layer]) == pytest.approx(buf, rel=1e-12)
    kept = co.expansion_plan(cc.STEP2, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, M=cc.M, C1=cc.C1, pruner=pr)
    assert kept == cc.KEPT2
    for layer, a in cc.ALPHA_AFTER_2.items():
        assert pr.alpha(layer) == pytest.approx(a, rel=1e-12)
    for layer, buf in cc.BUFFERS_AFTER_2.items():
        assert list(pr.A[layer]) == pytest.approx(buf, rel=1e-12)
    # the same second step on fresh buffers goes one layer further: the stop came from A_2's content
    fresh = co.expansion_plan(cc.STEP2, cc.S_D, cc.S_T, n0=cc.N0, L=cc.L, M=cc.M, C1=cc.C1,
                              pruner=co.DepthPruner(R=cc.R, C2=cc.C2))
    assert fresh == [3, 2, 2]
