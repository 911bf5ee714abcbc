"""CPU oracle of the cost-aware tree-size selection (CAST) host logic.

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product path).  Plain
Python in double precision, each function written from what the paper defines, in the paper's
notation; no blocking, no shortcuts.  Shares no code with the native implementation.

What is written out here (paper, section "Method"):
  * the lookup-table row selector select(c)                     (Method, 2nd paragraph)
  * the cumulative utility u_k of a layer                       (Eq. 1)
  * the normalised cost c_k of a layer                          (Eq. 2)
  * "Select Maximum Valid Index"                                (Algorithm 1)
  * breadth pruning = Algorithm 1 on (u, c) with threshold C1   (Dynamic Expansion Stage)
  * depth pruning with the FIFO buffers A_i and threshold C2    (Dynamic Expansion Stage, last paragraph)
  * the number of nodes to verify, threshold C3                 (Dynamic Reranking Stage)
  * keeping the top-scoring nodes as a subtree                  (Tree Reranking Phase)

Readings taken where the text is garbled or silent:
  * select(c): printed with max(.), which would always return the last table row; read as
    min(floor(c / L), M - 1) + 1 rows of L, i.e. the first grid point above c, clamped to M*L.
  * Cost tables are indexed [row of select(c)][n] with n = 1..N (1-based, as printed).
  * The batch-averaged score of the reranking stage is the rank-wise mean of the per-sample
    scores sorted in descending order (the same averaging as Eq. 1).
  * Pins: the paper prints no numeric example of these functions, so no expected value is taken from it; they
    are pinned (tests/test_cast_oracle_pins.py) by the paper's theorem, by closed forms, by limits and
    monotonicity, and by cases worked by hand.
"""
from __future__ import annotations

from collections import deque
from typing import List, Sequence


def select_context(c: int, L: int, M: int) -> int:
    """Table row (as a context length, a multiple of L) used for a context of c tokens."""
    return (min(c // L, M - 1) + 1) * L


def select_max_valid_index(u: Sequence[float], c: Sequence[float], C: float) -> int:
    """Algorithm 1, from what it defines.  u, c of equal length n >= 1, c strictly increasing.
    Index j (1-based) is valid iff no chord that ends in it is too flat: the smallest slope
    (u[j]-u[i]) / (c[j]-c[i]) over the earlier indices i < j is at least C (index 1 has no
    chord and is always valid).  The result is the largest valid index."""
    def flattest_chord_into(j: int) -> float:
        slopes = [(float(u[j]) - float(u[i])) / (float(c[j]) - float(c[i])) for i in range(j)]
        return min(slopes) if slopes else float("inf")

    valid = [j + 1 for j in range(len(u)) if not flattest_chord_into(j) < C]
    return valid[-1]


def layer_utility(scores: Sequence[Sequence[float]]) -> List[float]:
    """Eq. 1.  scores[j][s]: confidence of the s-th best candidate of sample j (descending per
    sample), all samples with the same number N_i of candidates.  Returns [u_1 .. u_{N_i}]."""
    B = len(scores)
    N = len(scores[0])
    u = []
    for k in range(1, N + 1):
        total = 0.0
        for j in range(B):
            for s in range(k):
                total += float(scores[j][s])
        u.append(total / B)
    return u


def layer_cost(S_D: Sequence[Sequence[float]], S_T: Sequence[Sequence[float]], ctx: int, L: int, M: int,
               n_candidates: int) -> List[float]:
    """Eq. 2.  S_D, S_T: tables of one batch size, row r-1 for context r*L (r = 1..M), column n-1 for
    n tokens.  Returns [c_1 .. c_{n_candidates}] = draft cost of k tokens over target cost of 1."""
    row = select_context(ctx, L, M) // L - 1
    return [float(S_D[row][k - 1]) / float(S_T[row][0]) for k in range(1, n_candidates + 1)]


def breadth_prune(scores, S_D, S_T, ctx: int, L: int, M: int, C1: float):
    """Number of nodes n_i kept in a layer, with the (u, c) pair at that index."""
    u = layer_utility(scores)
    c = layer_cost(S_D, S_T, ctx, L, M, len(u))
    n_i = select_max_valid_index(u, c, C1)
    return n_i, u[n_i - 1], c[n_i - 1]


class DepthPruner:
    """Buffers A_i (one per layer, first-in-first-out, at most R values, started with {1}) and the
    test that decides whether layer i+1 is generated."""

    def __init__(self, R: int, C2: float):
        self.R, self.C2 = R, C2
        self.A = {}

    def _buf(self, i: int) -> deque:
        if i not in self.A:
            self.A[i] = deque([1.0])
        return self.A[i]

    def alpha(self, i: int) -> float:
        buf = self._buf(i)
        return sum(buf) / len(buf)

    def should_expand(self, i: int, u_ni: float, c_ni: float) -> bool:
        return self.alpha(i) * u_ni / c_ni >= self.C2

    def update(self, i: int, u_next: float, u_cur: float) -> float:
        phi = u_next / u_cur
        buf = self._buf(i)
        buf.append(phi)
        while len(buf) > self.R:
            buf.popleft()
        return phi


def expansion_plan(layers, S_D, S_T, n0: int, L: int, M: int, C1: float, pruner: DepthPruner):
    """Runs breadth and depth pruning over the candidate layers in order.  layers[i] is the score
    matrix of layer i+1's candidates.  The context of layer i is n0 plus the nodes kept so far
    (n0 = 0 gives the printed formula).  Returns the kept node counts [n_1, n_2, ...]."""
    kept = []
    prev = None
    for idx, scores in enumerate(layers):
        i = idx + 1
        ctx = n0 + sum(kept)
        n_i, u_ni, c_ni = breadth_prune(scores, S_D, S_T, ctx, L, M, C1)
        kept.append(n_i)
        if prev is not None:
            pruner.update(i - 1, u_ni, prev)
        prev = u_ni
        if idx + 1 < len(layers) and not pruner.should_expand(i, u_ni, c_ni):
            break
    return kept


def rerank_count(tree_scores: Sequence[Sequence[float]], S_T, n0: int, L: int, M: int, m: int, C3: float) -> int:
    """Number of nodes handed to the target model.  tree_scores[j]: scores of all nodes of sample
    j's expanded tree (any order; every sample has the same number of nodes)."""
    B = len(tree_scores)
    ranked = [sorted((float(x) for x in row), reverse=True) for row in tree_scores]
    N = min(len(ranked[0]), m)
    v = [sum(ranked[j][s] for j in range(B)) / B for s in range(N)]
    u = []
    acc = 0.0
    for s in range(N):
        acc += v[s]
        u.append(acc)
    row = select_context(n0, L, M) // L - 1
    c = [float(S_T[row][k - 1]) / float(S_T[row][0]) for k in range(1, N + 1)]
    return select_max_valid_index(u, c, C3)


def select_subtree(score: Sequence[float], parent: Sequence[int], keep: int):
    """Keeps the `keep` best-scoring nodes (ties: lower index first) and relabels them in ascending
    original index.  Returns (old_index, new_parent).  Raises if the kept set is not closed under
    taking parents (cannot happen when a child's score never exceeds its parent's)."""
    n = len(score)
    order = sorted(range(n), key=lambda i: (-float(score[i]), i))
    kept = sorted(order[:keep])
    new_id = {old: new for new, old in enumerate(kept)}
    new_parent = []
    for old in kept:
        p = parent[old]
        if p < 0:
            new_parent.append(-1)
        else:
            if p not in new_id:
                raise ValueError("kept set is not closed under parents")
            new_parent.append(new_id[p])
    return kept, new_parent
