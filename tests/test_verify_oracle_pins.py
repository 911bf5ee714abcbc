"""Pins of oracle/verify_oracle.py (greedy tree acceptance, K/V commit) by other routes: the
all-edges-match characterisation of the accepted path computed per node without walking, the chain
tree as plain sequential speculative decoding at temperature 0, hand-made cases, and invariants of
the commit (rows written = rows of the path, everything else untouched).  CPU only."""
import numpy as np
import pytest

from oracle import verify_oracle as vo


def random_tree(rng, T, window=6):
    return np.array([-1] + [int(rng.integers(max(0, i - window), i)) for i in range(1, T)], np.int32)


def distinct_sibling_tokens(rng, parent, vocab=50):
    """Tokens such that the children of one node all differ (as the children of a draft node do)."""
    T = len(parent)
    tok = np.zeros(T, np.int32)
    used = {}
    for i in range(T):
        p = int(parent[i])
        while True:
            t = int(rng.integers(0, vocab))
            if t not in used.setdefault(p, set()):
                used[p].add(t)
                tok[i] = t
                break
    return tok


def test_accepted_path_is_the_deepest_node_whose_every_edge_matches():
    """With distinct sibling tokens, node i is accepted iff on its root path every node's token equals
    its parent's target token; those nodes form one chain and the walk ends at its deepest node."""
    rng = np.random.Generator(np.random.PCG64(21))
    for _ in range(200):
        T = int(rng.integers(1, 80))
        parent = random_tree(rng, T)
        draft = distinct_sibling_tokens(rng, parent)
        target = rng.integers(0, 50, T).astype(np.int32)
        for i in rng.integers(0, T, size=min(T, 12)):          # plant matches so that paths get long
            c = [j for j in range(T) if parent[j] == i]
            if c:
                target[i] = draft[c[int(rng.integers(0, len(c)))]]
        ok = np.zeros(T, bool)
        ok[0] = True
        for i in range(1, T):
            ok[i] = ok[parent[i]] and draft[i] == target[parent[i]]
        accepted = sorted(np.nonzero(ok)[0])
        paths, nxt = vo.accept_greedy(parent, [0, T], draft, target)
        assert paths[0] == accepted
        for a, b in zip(paths[0][:-1], paths[0][1:]):
            assert parent[b] == a
        assert nxt[0] == target[paths[0][-1]]


def test_chain_is_sequential_greedy_speculative_decoding():
    """A chain-shaped tree: accept drafted tokens while they equal the target's, emit the target's token at
    the first mismatch (or after the last token)."""
    rng = np.random.Generator(np.random.PCG64(22))
    for _ in range(100):
        T = int(rng.integers(1, 20))
        parent = np.arange(-1, T - 1, dtype=np.int32)
        draft = rng.integers(0, 4, T).astype(np.int32)
        target = rng.integers(0, 4, T).astype(np.int32)
        n = 1
        while n < T and draft[n] == target[n - 1]:
            n += 1
        paths, nxt = vo.accept_greedy(parent, [0, T], draft, target)
        assert paths[0] == list(range(n)) and nxt[0] == target[n - 1]


def test_hand_made_cases():
    #        0
    #      / | \
    #     1  2  3        tokens 7 8 9
    #    /|     |
    #   4 5     6        tokens 1 2 3
    parent = np.array([-1, 0, 0, 0, 1, 1, 3], np.int32)
    draft = np.array([0, 7, 8, 9, 1, 2, 3], np.int32)
    target = np.array([9, 0, 0, 3, 0, 0, 5], np.int32)          # root wants 9 -> node 3; node 3 wants 3 -> node 6
    assert vo.accept_greedy(parent, [0, 7], draft, target) == ([[0, 3, 6]], [5])
    target[0] = 4                                               # no child of the root carries 4
    assert vo.accept_greedy(parent, [0, 7], draft, target) == ([[0]], [4])
    target[0], target[1] = 7, 2                                 # 0 -> 1 -> 5, then node 5 has no children
    assert vo.accept_greedy(parent, [0, 7], draft, target) == ([[0, 1, 5]], [0])
    draft[2] = 7                                                # duplicate sibling token: the lower index wins
    assert vo.accept_greedy(parent, [0, 7], draft, target)[0] == [[0, 1, 5]]
    # batch with an empty tree and a single-node tree
    p2, n2 = vo.accept_greedy(np.array([-1], np.int32), [0, 0, 1], np.array([3], np.int32), np.array([8], np.int32))
    assert p2 == [[], [0]] and n2 == [-1, 8]


def test_commit_dense_and_paged_write_exactly_the_path_rows():
    rng = np.random.Generator(np.random.PCG64(23))
    B, Hkv, D = 3, 2, 8
    T = np.array([9, 1, 5])
    cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    cap = np.array([20, 6, 9])
    cu_L = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
    L = np.array([11, 5, 0], np.int32)
    kc = rng.integers(0, 2 ** 16, (cap.sum(), Hkv, D)).astype(np.uint16)
    vc = rng.integers(0, 2 ** 16, (cap.sum(), Hkv, D)).astype(np.uint16)
    kt = rng.integers(0, 2 ** 16, (T.sum(), Hkv, D)).astype(np.uint16)
    vt = rng.integers(0, 2 ** 16, (T.sum(), Hkv, D)).astype(np.uint16)
    paths = [[0, 2, 7], [0], [0, 1, 3, 4]]
    k2, v2, L2 = vo.commit_path_dense(kc, vc, cu_L, L, kt, vt, cu_T, paths)
    assert list(L2) == [14, 6, 4]
    touched = np.zeros(cap.sum(), bool)
    for b, path in enumerate(paths):
        for j, node in enumerate(path):
            row = cu_L[b] + L[b] + j
            touched[row] = True
            assert np.array_equal(k2[row], kt[cu_T[b] + node]) and np.array_equal(v2[row], vt[cu_T[b] + node])
    assert np.array_equal(k2[~touched], kc[~touched]) and np.array_equal(v2[~touched], vc[~touched])
    with pytest.raises(ValueError):
        vo.commit_path_dense(kc, vc, cu_L, np.array([18, 5, 0], np.int32), kt, vt, cu_T, paths)   # 18 + 3 > 20
    # paged: the same positions through a page table give the same rows
    ps, pages_per = 4, 6
    perm = rng.permutation(B * pages_per).reshape(B, pages_per).astype(np.int32)
    kp = np.zeros((B * pages_per, ps, Hkv, D), np.uint16)
    vp = np.zeros_like(kp)
    k3, v3, L3 = vo.commit_path_paged(kp, vp, perm, ps, L, kt, vt, cu_T, paths)
    assert list(L3) == [14, 6, 4]
    for b, path in enumerate(paths):
        for j, node in enumerate(path):
            t = L[b] + j
            assert np.array_equal(k3[perm[b, t // ps], t % ps], kt[cu_T[b] + node])
    assert int((k3 != 0).any(axis=(2, 3)).sum()) <= sum(len(p) for p in paths)
