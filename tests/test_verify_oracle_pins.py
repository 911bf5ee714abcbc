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


# ---- acceptance by speculative sampling (oracle: accept_sampling) ----

def dirichlet_rows(rng, n, V, conc=0.7):
    return rng.dirichlet(np.full(V, conc), size=n).astype(np.float32)


def test_sampling_on_a_chain_is_the_rule_of_the_paper_written_out():
    """A chain tree is plain speculative decoding (paper, Preliminary): token i is accepted iff
    u_i <= min(1, p_i / q_i); at the first rejection one token is drawn from norm(max(0, p - q)), after the last
    acceptance from p.  Written here with divisions and normalised vectors, not the oracle's way."""
    rng = np.random.Generator(np.random.PCG64(31))
    V = 11
    for _ in range(300):
        T = int(rng.integers(1, 9))
        parent = np.arange(-1, T - 1, dtype=np.int32)
        P, Q = dirichlet_rows(rng, T, V), dirichlet_rows(rng, T, V)
        tok = np.array([0] + [int(rng.choice(V, p=Q[i - 1].astype(np.float64) / Q[i - 1].astype(np.float64).sum()))
                              for i in range(1, T)], np.int32)
        u, uf = rng.random(T), rng.random(1)
        paths, nxt = vo.accept_sampling(parent, np.array([0, T], np.int32), tok, P, Q, u, uf)
        # the rule, directly
        n_acc, dist = 1, P[0].astype(np.float64)
        for i in range(1, T):
            p, q = P[i - 1].astype(np.float64), Q[i - 1].astype(np.float64)
            p, x = p / p.sum(), int(tok[i])
            if u[i] <= min(1.0, p[x] / q[x]):
                n_acc += 1
                dist = P[i].astype(np.float64)
            else:
                dist = np.maximum(0.0, p - q)
                break
        dist = dist / dist.sum()
        want = int(np.searchsorted(np.cumsum(dist), uf[0], side="right"))
        assert paths[0] == list(range(n_acc))
        # (the oracle keeps the residual in float32 and unnormalised: equal unless uf sits on a boundary)
        cs = np.cumsum(dist)
        if np.min(np.abs(cs - uf[0])) > 1e-6:
            assert nxt[0] == want


def test_sampling_emits_tokens_distributed_as_the_target():
    """The theorem the rule rests on (paper, Preliminary: the output is a sample of the target distribution):
    whatever q is, with k children drawn independently from q the first emitted token -- the accepted child's, or
    the one drawn from the last residual -- has distribution p.  200 000 seeded trials, 6-token vocabulary."""
    rng = np.random.Generator(np.random.PCG64(32))
    V, N, k = 6, 200000, 3
    p, q = dirichlet_rows(rng, 1, V)[0], dirichlet_rows(rng, 1, V)[0]
    parent = np.tile(np.array([-1] + [0] * k, np.int32), N)
    cu = (np.arange(N + 1) * (k + 1)).astype(np.int32)
    tok = np.zeros((N, k + 1), np.int32)
    tok[:, 1:] = rng.choice(V, size=(N, k), p=q.astype(np.float64) / q.astype(np.float64).sum())
    P, Q = np.tile(p, ((k + 1) * N, 1)), np.tile(q, ((k + 1) * N, 1))
    paths, nxt = vo.accept_sampling(parent, cu, tok.reshape(-1), P, Q, rng.random((k + 1) * N), rng.random(N))
    first = np.array([tok[i, pth[1]] if len(pth) > 1 else nxt[i] for i, pth in enumerate(paths)])
    freq = np.bincount(first, minlength=V) / N
    sigma = np.sqrt(p.astype(np.float64) * (1 - p.astype(np.float64)) / N)
    assert np.all(np.abs(freq - p) <= 5 * sigma + 1e-6), (freq, p)
    # and it is not trivially so: the children alone are distributed as q, visibly different from p
    assert np.abs(np.bincount(tok[:, 1], minlength=V) / N - p).max() > 20 * sigma.max()


def test_sampling_with_rows_taken_as_distributions():
    """Reading S5 (unit_rows: a freshly reached node's Z is 1, not the row's sum).  (a) On rows whose float32 entries
    add up to exactly one (multiples of 2^-12) the two readings are the same computation.  (b) On a chain it is the
    rule of the paper as printed -- u <= p(x) / q(x) with the rows as they are, no division by their sums, residual
    max(0, p - q) -- written out here.  (c) The theorem still holds: the first emitted token is distributed as p."""
    rng = np.random.Generator(np.random.PCG64(35))
    V = 9
    def dyadic_rows(n):
        cuts = np.sort(rng.integers(0, 4097, size=(n, V - 1)), axis=1)
        w = np.diff(np.concatenate([np.zeros((n, 1), np.int64), cuts, np.full((n, 1), 4096)], axis=1), axis=1)
        return (w / 4096.0).astype(np.float32)
    for _ in range(200):
        T = int(rng.integers(1, 9))
        parent = np.array([-1] + [int(rng.integers(0, i)) for i in range(1, T)], np.int32)
        P, Q = dyadic_rows(T), dirichlet_rows(rng, T, V)
        assert np.all(P.astype(np.float64).sum(axis=1) == 1.0)
        tok = rng.integers(0, V, T).astype(np.int32)
        u, uf, cu = rng.random(T), rng.random(1), np.array([0, T], np.int32)
        try:
            want = vo.accept_sampling(parent, cu, tok, P, Q, u, uf)
        except ValueError:
            continue
        assert vo.accept_sampling(parent, cu, tok, P, Q, u, uf, unit_rows=True) == want
    differs = 0
    for _ in range(300):
        T = int(rng.integers(1, 9))
        parent = np.arange(-1, T - 1, dtype=np.int32)
        # (rows that sum to 0.7: the reading must not look at their sums, and the default reading decides otherwise)
        P, Q = (0.7 * dirichlet_rows(rng, T, V)).astype(np.float32), dirichlet_rows(rng, T, V)
        tok = np.array([0] + [int(rng.choice(V, p=Q[i - 1].astype(np.float64) / Q[i - 1].astype(np.float64).sum()))
                              for i in range(1, T)], np.int32)
        u, uf = rng.random(T), rng.random(1)
        try:
            paths, nxt = vo.accept_sampling(parent, np.array([0, T], np.int32), tok, P, Q, u, uf, unit_rows=True)
        except ValueError:
            continue
        differs += vo.accept_sampling(parent, np.array([0, T], np.int32), tok, P, Q, u, uf)[0] != paths
        n_acc, dist = 1, P[0].astype(np.float64)
        for i in range(1, T):
            p, q, x = P[i - 1].astype(np.float64), Q[i - 1].astype(np.float64), int(tok[i])
            if u[i] <= min(1.0, p[x] / q[x]):
                n_acc += 1
                dist = P[i].astype(np.float64)
            else:
                dist = np.maximum(0.0, p - q)
                break
        assert paths[0] == list(range(n_acc))
        cs = np.cumsum(dist / dist.sum())
        if np.min(np.abs(cs - uf[0])) > 1e-6:
            assert nxt[0] == int(np.searchsorted(cs, uf[0], side="right"))
    assert differs > 20
    N, k, V = 100000, 3, 6
    p, q = dirichlet_rows(rng, 1, V)[0], dirichlet_rows(rng, 1, V)[0]
    parent = np.tile(np.array([-1] + [0] * k, np.int32), N)
    cu = (np.arange(N + 1) * (k + 1)).astype(np.int32)
    tok = np.zeros((N, k + 1), np.int32)
    tok[:, 1:] = rng.choice(V, size=(N, k), p=q.astype(np.float64) / q.astype(np.float64).sum())
    P, Q = np.tile(p, ((k + 1) * N, 1)), np.tile(q, ((k + 1) * N, 1))
    paths, nxt = vo.accept_sampling(parent, cu, tok.reshape(-1), P, Q, rng.random((k + 1) * N), rng.random(N), unit_rows=True)
    first = np.array([tok[i, pth[1]] if len(pth) > 1 else nxt[i] for i, pth in enumerate(paths)])
    freq = np.bincount(first, minlength=V) / N
    sigma = np.sqrt(p.astype(np.float64) * (1 - p.astype(np.float64)) / N)
    assert np.all(np.abs(freq - p) <= 5 * sigma + 1e-6), (freq, p)


def test_sampling_special_cases():
    rng = np.random.Generator(np.random.PCG64(33))
    V = 9
    for _ in range(100):
        T = int(rng.integers(2, 30))
        parent = random_tree(rng, T)
        # (token V - 1 is never drafted)
        tok = distinct_sibling_tokens(rng, parent, vocab=V - 1) if T < 8 else rng.integers(0, V - 1, T).astype(np.int32)
        cu = np.array([0, T], np.int32)
        P = dirichlet_rows(rng, T, V)
        u, uf = rng.random(T), rng.random(1)
        # q = p: the ratio is 1, so the first child of every node on the way is accepted for any u < 1
        paths, _ = vo.accept_sampling(parent, cu, tok, P, P, np.full(T, 0.999), uf)
        cur, want = 0, [0]
        while True:
            first = [c for c in range(cur + 1, T) if parent[c] == cur][:1]
            if not first:
                break
            cur = first[0]
            want.append(cur)
        assert paths[0] == want
        # a point-mass target (temperature 0) makes it the greedy rule: the child carrying the target's token
        target = rng.integers(0, V - 1, T).astype(np.int32)
        for i in rng.integers(0, T, size=6):
            if parent[i] >= 0:
                target[parent[i]] = tok[i]
        onehot = np.zeros((T, V), np.float32)
        onehot[np.arange(T), target] = 1.0
        Q = dirichlet_rows(rng, T, V, conc=2.0)
        gp, gn = vo.accept_greedy(parent, cu, tok, target)
        sp, sn = vo.accept_sampling(parent, cu, tok, onehot, Q, u, uf)
        assert sp == gp and sn == gn
        # a token the target gives no probability is never accepted, even with u = 0
        Pz = P.copy()
        Pz[:, np.unique(tok)] = 0.0                              # no drafted token has target mass anywhere
        zp, _ = vo.accept_sampling(parent, cu, tok, Pz, dirichlet_rows(rng, T, V), np.zeros(T), uf)
        assert zp == [[0]]
        # max_path is an interface limit
        lp, _ = vo.accept_sampling(parent, cu, tok, P, P, np.zeros(T), uf, max_path=2)
        assert len(lp[0]) <= 2
