"""Pins of oracle/draft_oracle.py (one layer of draft-tree expansion) by other routes: selection written as a
repeated search for the maximum, numpy's own argmax / sort on tie-free rows, the product definition of a node's
value (paper, Tree Expansion Phase), and the property the Tree Reranking Phase relies on.  CPU only."""
import numpy as np
import pytest

from oracle import cast_oracle as co
from oracle import draft_oracle as do


def log_softmax_rows(rng, n, V, scale=3.0):
    z = rng.standard_normal((n, V)) * scale
    z = z - z.max(axis=1, keepdims=True)
    return (z - np.log(np.exp(z).sum(axis=1, keepdims=True))).astype(np.float32)


def test_selection_is_a_repeated_search_for_the_maximum():
    """K times: take the largest remaining log-probability of the row (the first one among equals); then, over all
    candidates of a sequence, the same with the scores.  Values drawn from a handful of levels, so ties abound."""
    rng = np.random.Generator(np.random.PCG64(41))
    for _ in range(60):
        B, V, K = int(rng.integers(1, 4)), int(rng.integers(3, 40)), int(rng.integers(1, 4))
        K = min(K, V)
        n = rng.integers(0, 5, B)
        cu = np.concatenate([[0], np.cumsum(n)]).astype(np.int32)
        logp = (-rng.integers(0, 6, (int(cu[-1]), V)) * 0.25).astype(np.float32)
        score = (-rng.integers(0, 4, int(cu[-1])) * 0.5).astype(np.float32)
        got = do.expand_layer(score, cu, logp, K)
        for b in range(B):
            cand = []
            for r in range(int(cu[b]), int(cu[b + 1])):
                left = list(range(V))
                for _k in range(K):
                    best = left[0]
                    for t in left:
                        if logp[r, t] > logp[r, best]:
                            best = t
                    left.remove(best)
                    cand.append((np.float32(score[r] + logp[r, best]), r - int(cu[b]), best))
            want = []
            while cand:
                best = 0
                for i in range(len(cand)):
                    if cand[i][0] > cand[best][0]:
                        best = i
                want.append(cand.pop(best))
            cs, cp, ct = got[b]
            assert [float(x) for x in cs] == [float(w[0]) for w in want]
            assert list(cp) == [w[1] for w in want] and list(ct) == [w[2] for w in want]


def test_tie_free_rows_against_numpy_sort_and_argmax():
    rng = np.random.Generator(np.random.PCG64(42))
    n, V, K = 7, 5000, 10
    logp = np.stack([-(rng.permutation(V) + 1) * 0.001 for _ in range(n)]).astype(np.float32)   # no two equal in a row
    assert all(len(np.unique(logp[r])) == V for r in range(n))
    score = -rng.random(n).astype(np.float32)
    (cs, cp, ct), = do.expand_layer(score, [0, n], logp, K)
    # the tokens kept under each row are numpy's K largest, and K = 1 is argmax
    for r in range(n):
        assert sorted(ct[cp == r]) == sorted(np.argsort(logp[r])[-K:])
    (cs1, cp1, ct1), = do.expand_layer(score, [0, n], logp, 1)
    assert sorted(zip(cp1, ct1)) == [(r, int(np.argmax(logp[r]))) for r in range(n)]
    # the scores are all the children's scores, sorted
    allc = np.sort((score[:, None] + np.sort(logp, axis=1)[:, -K:]).astype(np.float32).ravel())[::-1]
    assert np.array_equal(cs, allc)
    assert np.all(np.diff(cs.astype(np.float64)) <= 0)


def grow(rng, V, K, depth, keep):
    """A tree grown layer by layer from the root (score 0 = log 1): each layer expands the `keep` best candidates of
    the layer before.  Returns (parent, token, score, p_edge) over all nodes, root first."""
    parent, token, score, p_edge = [-1], [0], [np.float32(0.0)], [1.0]
    layer = [0]
    for _d in range(depth):
        logp = log_softmax_rows(rng, len(layer), V)
        (cs, cp, ct), = do.expand_layer(np.array([score[i] for i in layer], np.float32), [0, len(layer)], logp, K)
        nxt = []
        for s, p, t in list(zip(cs, cp, ct))[:keep]:
            parent.append(layer[p]); token.append(int(t)); score.append(np.float32(s))
            p_edge.append(float(np.exp(np.float64(logp[p, t]))))
            nxt.append(len(parent) - 1)
        layer = nxt
    return parent, token, score, p_edge


def test_scores_are_logs_of_the_products_along_the_paths():
    """v(u) = product of P_D over the path of u, the root 1 (paper, Tree Expansion Phase)."""
    rng = np.random.Generator(np.random.PCG64(43))
    parent, token, score, p_edge = grow(rng, V=300, K=4, depth=6, keep=5)
    for i in range(len(parent)):
        v, j = 1.0, i
        while j >= 0:
            v *= p_edge[j]
            j = parent[j]
        assert np.exp(np.float64(score[i])) == pytest.approx(v, rel=2e-6)


def test_best_nodes_of_a_grown_tree_form_a_subtree():
    """A child's value never exceeds its parent's, so keeping the m best nodes keeps every kept node's parent (paper,
    Tree Reranking Phase); with the sign of the log-probabilities flipped that fails, so the check has teeth."""
    rng = np.random.Generator(np.random.PCG64(44))
    for _ in range(20):
        parent, token, score, _ = grow(rng, V=200, K=3, depth=5, keep=4)
        for i in range(1, len(parent)):
            assert score[i] <= score[parent[i]]
        for m in (1, 5, len(parent) // 2, len(parent)):
            old, newp = co.select_subtree(score, parent, m)
            assert len(old) == m and all(p < i for i, p in enumerate(newp))
    flipped = [np.float32(-s) for s in score]
    with pytest.raises(ValueError):
        co.select_subtree(flipped, parent, len(parent) // 2)


def test_degenerate_inputs():
    logp = np.full((2, 6), -np.inf, np.float32)
    logp[0, 4] = 0.0                                 # a point mass: one real child, the rest have value 0
    logp[1, :] = np.float32(np.log(1 / 6))            # a uniform row: the first K tokens
    out = do.expand_layer(np.array([0.0, -1.0], np.float32), [0, 1, 2, 2], logp, 3)
    cs, cp, ct = out[0]
    assert list(ct) == [4, 0, 1] and cs[0] == 0.0 and np.all(np.isneginf(cs[1:]))
    cs, cp, ct = out[1]
    assert list(ct) == [0, 1, 2] and np.all(cs == np.float32(np.float32(-1.0) + np.float32(np.log(1 / 6))))
    assert len(out[2][0]) == 0                        # a sequence without rows
