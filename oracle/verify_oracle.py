"""CPU oracle of the steps that close a verification pass after the attention: acceptance of a root
path of the draft tree (greedy, temperature 0; and by speculative sampling, accept_sampling below), and the
commit of the accepted nodes' K/V rows to the end of the sequence's cache.

TEST INFRASTRUCTURE ONLY: imported by tests/ (nothing in the product path).  Plain numpy /
Python loops; shares no code with the HIP kernels.

Acceptance (paper, Preliminary: "Speculative Decoding" -- a drafted token is accepted with
probability min(1, p/q), else the target's own token is taken -- and "EAGLE": the draft is a tree
and a rejected token leaves its siblings' subtrees in play).  At temperature 0 the target
distribution is a point mass on its argmax, so p/q is 1/q >= 1 for the drafted token that equals
the argmax and 0 for every other: the walk goes from the root to the child whose drafted token
equals the target's argmax at the current node, and stops where no child does; the target's argmax
at the last accepted node is the next (bonus) token.

Readings: node 0 is the root and is always accepted (it is the token the previous step emitted);
nodes are in topological order; when several children carry the matching token the lowest index is
taken (a draft tree's siblings are distinct tokens, so this does not arise in practice); other roots
of a forest are unreachable.  Commit: accepted node j of sequence b (in path order) goes to cache
position L_b + j; nothing else in the cache changes.
Pins: the paper prints no numeric example of either step, so no expected value is taken from it; the pins
are definitions by another route (all-edges-match characterisation, brute force) and invariants.
"""
from __future__ import annotations

import numpy as np


def accept_greedy(parent, cu_T, draft_token, target_token, max_path=None):
    """parent, draft_token, target_token: int arrays [sum_T] (parent local to its tree, -1 = root);
    target_token[i] = the target model's argmax for the position after node i.
    Returns (paths: list of lists of local node indices, next_token: list).  With max_path the walk
    also ends once that many nodes are accepted (an interface limit, not part of the method)."""
    B = len(cu_T) - 1
    paths, nxt = [], []
    for b in range(B):
        t0, T = int(cu_T[b]), int(cu_T[b + 1] - cu_T[b])
        if T == 0:
            paths.append([])
            nxt.append(-1)
            continue
        cur = 0
        path = [0]
        while max_path is None or len(path) < max_path:
            want = int(target_token[t0 + cur])
            found = -1
            for c in range(cur + 1, T):
                if int(parent[t0 + c]) == cur and int(draft_token[t0 + c]) == want:
                    found = c
                    break
            if found < 0:
                break
            cur = found
            path.append(cur)
        paths.append(path)
        nxt.append(int(target_token[t0 + cur]))
    return paths, nxt


def accept_sampling(parent, cu_T, draft_token, p_target, q_draft, u, u_final, max_path=None, unit_rows=False):
    """Acceptance by speculative sampling on draft trees (paper, Preliminary, "Speculative Decoding": a drafted
    token x with draft probability q(x) and target probability p(x) is accepted when a uniform number is at most
    min(1, p(x) / q(x)); after a rejection the target distribution is replaced by the residual norm(max(0, p - q));
    "EAGLE": with a tree draft a rejected token leaves its siblings in play).

    p_target[i], q_draft[i]: float32 [V] rows per node i -- the target's distribution of the token after node
    i's path, and the draft distribution node i's children were drawn from.  u[i]: the uniform number used when
    node i is tested as a child; u_final[b]: the one that draws the step's last token.  The walk starts at node 0
    (accepted).  At the current node the children are tested in index order against the current residual r
    (r = p at first); the first accepted child becomes the current node, with a fresh r; when every child is
    rejected, or there is none, or max_path nodes are accepted, one token is drawn from r / sum(r) and the walk
    ends.  Returns (paths, next_token).

    Readings (the paper states the rule for a chain only):
      S1  a child is tested against the residual left by its rejected elder siblings;
      S2  a rejection does not change q (the children of a node are independent draws from it), so the
          residual after a rejection is norm(max(0, r - q)) with the same q every time;
      S3  "u <= min(1, p/q)" is evaluated without a division as  r[x] > 0  and  u * q[x] * Z <= r[x],
          r kept unnormalised with Z = sum(r) (a token the draft gave probability 0 but the residual does not
          is accepted);
      S4  the last token is the smallest v whose cumulative weight r[0] + .. + r[v] exceeds u_final * Z
          (the last v with r[v] > 0 if rounding leaves none);
      S5  unit_rows: the caller states that every target row is a distribution (sums to one), and at a node that
          has just been reached Z is taken as 1 instead of being summed: the test is then u q(x) <= p(x) and the
          first residual max(0, p - q), both as the paper prints them.  The last draw still divides by the sum of what
          it draws from.
    Precision: r is held in float32 as the kernel holds it; sums, products and comparisons in float64.
    Pins: the paper prints no example; pinned by the chain rule written out, by the theorem that the emitted
    token is distributed as p, and by the temperature-0 and q = p special cases."""
    B = len(cu_T) - 1
    paths, nxt = [], []
    for b in range(B):
        t0, T = int(cu_T[b]), int(cu_T[b + 1] - cu_T[b])
        if T == 0:
            paths.append([])
            nxt.append(-1)
            continue
        cur, path = 0, [0]
        while True:
            r = np.array(p_target[t0 + cur], dtype=np.float32, copy=True)
            Z = 1.0 if unit_rows else float(r.astype(np.float64).sum())
            fresh = True
            q = np.asarray(q_draft[t0 + cur], dtype=np.float32).astype(np.float64)
            accepted = False
            if max_path is None or len(path) < max_path:
                for c in range(cur + 1, T):
                    if int(parent[t0 + c]) != cur:
                        continue
                    x = int(draft_token[t0 + c])
                    rx = float(r[x])
                    if rx > 0.0 and float(u[t0 + c]) * float(q[x]) * Z <= rx:
                        cur = c
                        path.append(c)
                        accepted = True
                        break
                    r_new = np.maximum(0.0, r.astype(np.float64) - Z * q).astype(np.float32)
                    Z_new = float(r_new.astype(np.float64).sum())
                    if not Z_new > 0.0:
                        raise ValueError("residual vanished: q is not a distribution the child could have been drawn from")
                    r, Z, fresh = r_new, Z_new, False
            if accepted:
                continue
            if fresh:
                Z = float(r.astype(np.float64).sum())          # (S5: the last draw is from r / sum(r) in either reading)
            cs = np.cumsum(r.astype(np.float64))
            hit = np.nonzero(cs > float(u_final[b]) * Z)[0]
            v = int(hit[0]) if len(hit) else int(np.nonzero(r > 0)[0][-1])
            paths.append(path)
            nxt.append(v)
            break
    return paths, nxt


def commit_path_dense(k_cache, v_cache, cu_L, L, k_tree, v_tree, cu_T, paths):
    """Dense ragged cache [sum_cap, Hkv, D] whose sequence b owns rows cu_L[b] .. cu_L[b+1]-1 and
    uses the first L[b]; returns (new k_cache, new v_cache, new L).  Raises if a sequence lacks room."""
    k, v = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    L_new = np.array(L, copy=True)
    for b, path in enumerate(paths):
        cap = int(cu_L[b + 1] - cu_L[b])
        if int(L[b]) + len(path) > cap:
            raise ValueError("no room in the cache of sequence %d" % b)
        for j, node in enumerate(path):
            row = int(cu_L[b]) + int(L[b]) + j
            k[row] = k_tree[int(cu_T[b]) + node]
            v[row] = v_tree[int(cu_T[b]) + node]
        L_new[b] = int(L[b]) + len(path)
    return k, v, L_new


def commit_path_paged(k_pool, v_pool, page_table, page_size, L, k_tree, v_tree, cu_T, paths):
    """Paged cache [pages, page_size, Hkv, D]; position t of sequence b is slot t % page_size of page
    page_table[b, t // page_size]."""
    k, v = np.array(k_pool, copy=True), np.array(v_pool, copy=True)
    L_new = np.array(L, copy=True)
    for b, path in enumerate(paths):
        for j, node in enumerate(path):
            t = int(L[b]) + j
            page = int(page_table[b, t // page_size])
            k[page, t % page_size] = k_tree[int(cu_T[b]) + node]
            v[page, t % page_size] = v_tree[int(cu_T[b]) + node]
        L_new[b] = int(L[b]) + len(path)
    return k, v, L_new
