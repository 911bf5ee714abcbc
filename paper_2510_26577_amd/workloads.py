"""Seeded synthetic inputs for tree-masked verification attention.

This module only *draws inputs*: cached lengths, draft trees (as parent arrays),
page tables and bf16 Q/K/V tensors.  It contains none of the method's
arithmetic (no mask construction, no softmax, no attention) so that the CPU
oracle and the HIP path can both consume exactly the same arrays without
sharing any code of the method itself.

The shapes follow the workloads of the paper's experiments (Experiments section and
the appendix "More Implementation Details": batch 1..32, at most 72 verified
tokens, tree depth up to 13, Llama-class 8B / 70B attention heads).  The
paper's benchmark prompts and trained models are not needed: the attention
path's cost and result depend on shapes and values only, so N(0,1) values
rounded once to bf16 stand in for real activations.

bf16 tensors are carried as ``numpy.uint16`` bit patterns (numpy has no bf16).
"""
from __future__ import annotations

import dataclasses
from typing import List, Optional

import numpy as np

BASE_SEED = 251026577


# ----------------------------------------------------------------------------
# bf16 helpers (storage format only)
# ----------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returned as uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = u + 0x7FFF + ((u >> 16) & 1)
    return (u >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Widen bf16 bit patterns exactly to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


# ----------------------------------------------------------------------------
# 8-bit floating point (OCP E4M3) storage of K/V: input preparation only
# ----------------------------------------------------------------------------
def _e4m3_magnitudes() -> np.ndarray:
    """The 127 finite magnitudes in code order (code c -> value), float32."""
    c = np.arange(127)
    e, m = c >> 3, c & 7
    return np.where(e == 0, m * 2.0 ** -9, (8 + m) * 2.0 ** (e - 10.0)).astype(np.float32)


def f32_to_e4m3(x: np.ndarray) -> np.ndarray:
    """Nearest finite E4M3 code of every element (ties to the even code, saturating at +-448), uint8."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    mags = _e4m3_magnitudes()
    out = np.empty(x.shape, np.uint8)
    flat_in, flat_out = x.reshape(-1), out.reshape(-1)
    step = 1 << 22
    for s in range(0, flat_in.size, step):
        v = flat_in[s:s + step]
        a = np.minimum(np.abs(v), mags[-1])
        hi = np.clip(np.searchsorted(mags, a), 1, 126)
        lo = hi - 1
        d_lo, d_hi = a - mags[lo], mags[hi] - a
        pick_hi = (d_hi < d_lo) | ((d_hi == d_lo) & (hi % 2 == 0))
        code = np.where(pick_hi, hi, lo).astype(np.uint8)
        flat_out[s:s + step] = code | (np.signbit(v).astype(np.uint8) << 7)
    return out


def to_fp8_kv(w: "Workload"):
    """The same workload with K and V (cache and tree) stored as E4M3 bytes, each tensor pair scaled so
    that its largest magnitude maps to 448.  Returns (workload with uint8 K/V, k_scale, v_scale)."""
    def amax(*arrs):
        m = max((float(np.abs(bf16_bits_to_f32(a)).max()) for a in arrs if a.size), default=1.0)
        return m if m > 0 else 1.0
    k_scale = amax(w.k_cache, w.k_tree) / 448.0
    v_scale = amax(w.v_cache, w.v_tree) / 448.0
    q8 = lambda a, sc: f32_to_e4m3(bf16_bits_to_f32(a) / np.float32(sc))
    w8 = dataclasses.replace(w, name=w.name + "_fp8kv", k_cache=q8(w.k_cache, k_scale), v_cache=q8(w.v_cache, v_scale),
                             k_tree=q8(w.k_tree, k_scale), v_tree=q8(w.v_tree, v_scale))
    return w8, k_scale, v_scale


def _normal_bf16(rng: np.random.Generator, shape) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24  # bound the float32 temporary
    for s in range(0, n, step):
        e = min(n, s + step)
        out[s:e] = f32_to_bf16_bits(rng.standard_normal(e - s, dtype=np.float32))
    return out.reshape(shape)


# ----------------------------------------------------------------------------
# draft-tree generators: each returns a parent array with parent[0] = -1 and
# parent[i] < i (topological order); depth is counted in edges, root = 0
# ----------------------------------------------------------------------------
def tree_window(rng: np.random.Generator, T: int, window: int = 3, max_depth: int = 4) -> np.ndarray:
    """parent[i] uniform in [max(0, i-window), i-1]; a draw that would exceed
    max_depth is redrawn among the window's shallow-enough nodes, the window
    widening downward when it has none."""
    parent = np.full(T, -1, dtype=np.int32)
    depth = np.zeros(T, dtype=np.int64)
    for i in range(1, T):
        lo = max(0, i - window)
        while True:
            cand = [j for j in range(lo, i) if depth[j] < max_depth]
            if cand:
                break
            lo -= 1
        j = int(cand[int(rng.integers(0, len(cand)))])
        parent[i] = j
        depth[i] = depth[j] + 1
    return parent


def tree_uniform(rng: np.random.Generator, T: int, max_depth: int) -> np.ndarray:
    """parent[i] uniform over earlier nodes whose depth is below max_depth."""
    parent = np.full(T, -1, dtype=np.int32)
    depth = np.zeros(T, dtype=np.int64)
    for i in range(1, T):
        cand = np.flatnonzero(depth[:i] < max_depth)
        j = int(cand[int(rng.integers(0, len(cand)))])
        parent[i] = j
        depth[i] = depth[j] + 1
    return parent


def tree_expand_prune(rng: np.random.Generator, T: int, depth: int = 6, max_branch: int = 4) -> np.ndarray:
    """Expansion-then-rerank shaped tree (Tree Expansion / Tree Reranking
    phases): breadth-first growth to `depth` with 1..max_branch children per
    node, child score = parent score * U(0,1) (so a child never outscores its
    parent), then the T best-scoring nodes are kept (ties -> lower index),
    which is therefore parent-closed, and relabelled in ascending original
    index so parent < child."""
    while True:
        par: List[int] = [-1]
        score: List[float] = [1.0]
        frontier = [0]
        for _ in range(depth):
            nxt = []
            for u in frontier:
                nc = int(rng.integers(1, max_branch + 1))
                for _c in range(nc):
                    par.append(u)
                    score.append(score[u] * float(rng.random()))
                    nxt.append(len(par) - 1)
            frontier = nxt
        if len(par) >= T:
            break
    score_a = np.asarray(score)
    order = np.lexsort((np.arange(len(par)), -score_a))  # by score desc, then index asc
    keep = np.sort(order[:T])
    new_id = {int(o): n for n, o in enumerate(keep)}
    out = np.full(T, -1, dtype=np.int32)
    for n, o in enumerate(keep):
        p = par[int(o)]
        out[n] = -1 if p < 0 else new_id[p]
    return out


def tree_chain(T: int) -> np.ndarray:
    return np.arange(-1, T - 1, dtype=np.int32)


def tree_star(T: int) -> np.ndarray:
    p = np.zeros(T, dtype=np.int32)
    p[0] = -1
    return p


def sampling_inputs(rng: np.random.Generator, parent: np.ndarray, cu_T: np.ndarray, V: int, temperature: float = 1.0,
                    drift: float = 1.0):
    """Inputs of acceptance by speculative sampling for given trees: per node a target distribution and a draft
    distribution over V tokens (softmax of normal logits divided by `temperature`; the draft's logits are the
    target's plus normal noise of standard deviation `drift`, so the two are as close as a draft model's are),
    the token of every non-root node drawn from its parent's draft distribution (siblings independently, as the
    paper's EAGLE-style drafts are read here), and the uniform numbers.
    Returns (p_target f32 [sum_T, V], q_draft f32 [sum_T, V], draft_token i32 [sum_T], u f32 [sum_T], u_final f32 [B])."""
    sum_T, B = int(cu_T[-1]), len(cu_T) - 1
    logit = rng.standard_normal((sum_T, V)) * 3.0
    def softmax(z):
        z = z / temperature
        e = np.exp(z - z.max(axis=1, keepdims=True))
        return (e / e.sum(axis=1, keepdims=True)).astype(np.float32)
    p = softmax(logit)
    q = softmax(logit + drift * rng.standard_normal((sum_T, V)))
    tok = np.zeros(sum_T, np.int32)
    for b in range(B):
        t0, T = int(cu_T[b]), int(cu_T[b + 1] - cu_T[b])
        for i in range(1, T):
            row = q[t0 + int(parent[t0 + i])].astype(np.float64)
            tok[t0 + i] = int(rng.choice(V, p=row / row.sum()))
    u = rng.random(sum_T, dtype=np.float32)
    u_final = rng.random(B, dtype=np.float32)
    return p, q, tok, u, u_final


def expansion_inputs(rng: np.random.Generator, n_rows, V: int, temperature: float = 1.0, levels: int = 0):
    """Inputs of one layer of draft-tree expansion: for every selected node (n_rows[b] of them in sequence b) its
    score (the log of its value: minus a sum of a few exponential draws) and the draft head's log-probabilities over
    V tokens (log-softmax of normal logits of standard deviation 3 / temperature; with levels > 0 the logits are
    rounded to that many distinct values, so that equal log-probabilities abound).
    Returns (cu_N i32 [B+1], score f32 [sum_N], logp f32 [sum_N, V])."""
    cu_N = np.concatenate([[0], np.cumsum(n_rows)]).astype(np.int32)
    sum_N = int(cu_N[-1])
    z = rng.standard_normal((sum_N, V)) * (3.0 / temperature)
    if levels > 0:
        z = np.round(z * levels / 12.0) * (12.0 / levels)
    z = z - z.max(axis=1, keepdims=True) if sum_N else z
    logp = (z - np.log(np.exp(z).sum(axis=1, keepdims=True))).astype(np.float32) if sum_N else z.astype(np.float32)
    score = (-rng.exponential(1.0, (sum_N, 3)).sum(axis=1)).astype(np.float32)
    return cu_N, score, logp


# ----------------------------------------------------------------------------
# workload container
# ----------------------------------------------------------------------------
@dataclasses.dataclass
class Workload:
    """One batch of tree-verification attention inputs (host arrays).

    Tensor layouts (innermost dimension contiguous):
      q              uint16 [sum_T, Hq,  D]   bf16 bits
      k_tree,v_tree  uint16 [sum_T, Hkv, D]
      dense cache:   k_cache,v_cache uint16 [sum_L, Hkv, D], cu_L int32 [B+1]
      paged cache:   k_cache,v_cache uint16 [n_pages, page_size, Hkv, D],
                     page_table int32 [B, max_pages]
      parent         int32 [sum_T]  per-tree local parent index, -1 for a root
      cu_T           int32 [B+1];   L int32 [B]
    """
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    scale: float
    T: np.ndarray
    cu_T: np.ndarray
    L: np.ndarray
    parent: np.ndarray
    q: np.ndarray
    k_tree: np.ndarray
    v_tree: np.ndarray
    k_cache: np.ndarray
    v_cache: np.ndarray
    cu_L: Optional[np.ndarray] = None
    page_table: Optional[np.ndarray] = None
    page_size: int = 0

    @property
    def paged(self) -> bool:
        return self.page_table is not None

    @property
    def sum_T(self) -> int:
        return int(self.cu_T[-1])

    @property
    def max_T(self) -> int:
        return int(self.T.max()) if self.B else 0

    @property
    def max_L(self) -> int:
        return int(self.L.max()) if self.B else 0

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    # --- byte / flop accounting used by the benchmark (definitions only) ---
    def kv_bytes(self) -> int:
        per_tok = 2 * self.Hkv * self.D * self.k_cache.dtype.itemsize   # 2 bytes per element (bf16), 1 for E4M3
        return int((int(self.L.sum()) + self.sum_T) * per_tok)

    def algorithmic_bytes(self) -> int:
        W = (self.max_T + 63) // 64
        b = self.kv_bytes()
        b += self.sum_T * self.Hq * self.D * 2          # Q
        b += self.sum_T * self.Hq * self.D * 4          # O
        b += self.sum_T * self.Hq * 4                   # LSE
        b += self.sum_T * 8 * W                         # ancestor mask
        if self.paged:
            b += int(sum((int(l) + self.page_size - 1) // self.page_size for l in self.L)) * 4
        return int(b)

    def algorithmic_flops(self) -> int:
        return int(4 * self.Hq * self.D * sum(int(t) * (int(l) + int(t)) for t, l in zip(self.T, self.L)))


def make_workload(name: str, seed: int, B: int, Hq: int, Hkv: int, D: int,
                  L, trees: List[np.ndarray], page_size: int = 0,
                  pool_slack: float = 1.25, rng: Optional[np.random.Generator] = None,
                  scale: Optional[float] = None) -> Workload:
    """Assemble a workload from given lengths and parent arrays, drawing the
    page table (if paged) and then Q, K_tree, V_tree, K_cache, V_cache, in that
    order, from `rng` (or a fresh PCG64(seed))."""
    if rng is None:
        rng = np.random.Generator(np.random.PCG64(seed))
    L = np.asarray(L, dtype=np.int32).reshape(B)
    T = np.asarray([len(t) for t in trees], dtype=np.int32)
    cu_T = np.zeros(B + 1, dtype=np.int32)
    cu_T[1:] = np.cumsum(T)
    parent = (np.concatenate([np.asarray(t, dtype=np.int32) for t in trees])
              if B and int(cu_T[-1]) else np.zeros(0, dtype=np.int32))
    sum_T = int(cu_T[-1])
    page_table = None
    cu_L = None
    if page_size:
        npages_b = [(int(l) + page_size - 1) // page_size for l in L]
        total = int(sum(npages_b))
        pool = max(1, int(np.ceil(pool_slack * total)))
        perm = rng.permutation(pool).astype(np.int32)
        max_pages = max(1, max(npages_b) if npages_b else 1)
        page_table = np.full((B, max_pages), -1, dtype=np.int32)  # -1: never read
        o = 0
        for b, n in enumerate(npages_b):
            page_table[b, :n] = perm[o:o + n]
            o += n
    else:
        cu_L = np.zeros(B + 1, dtype=np.int32)
        cu_L[1:] = np.cumsum(L)
    q = _normal_bf16(rng, (sum_T, Hq, D))
    k_tree = _normal_bf16(rng, (sum_T, Hkv, D))
    v_tree = _normal_bf16(rng, (sum_T, Hkv, D))
    if page_size:
        k_cache = _normal_bf16(rng, (pool, page_size, Hkv, D))
        v_cache = _normal_bf16(rng, (pool, page_size, Hkv, D))
    else:
        k_cache = _normal_bf16(rng, (int(cu_L[-1]), Hkv, D))
        v_cache = _normal_bf16(rng, (int(cu_L[-1]), Hkv, D))
    return Workload(name=name, B=B, Hq=Hq, Hkv=Hkv, D=D,
                    scale=float(scale if scale is not None else 1.0 / np.sqrt(D)),
                    T=T, cu_T=cu_T, L=L, parent=parent, q=q, k_tree=k_tree, v_tree=v_tree,
                    k_cache=k_cache, v_cache=v_cache, cu_L=cu_L, page_table=page_table,
                    page_size=page_size)


# ----------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------
SWEEP = {1: 64, 4: 32, 16: 16, 64: 8}  # batch -> tree size, shrinking as a cost-aware builder would


def config1() -> Workload:
    """Tiny: B=1, Hq=Hkv=4, D=64, L=128, T=8 (window-3 parents, depth <= 4)."""
    seed = BASE_SEED + 1
    rng = np.random.Generator(np.random.PCG64(seed))
    trees = [tree_window(rng, 8, 3, 4)]
    return make_workload("cfg1_tiny", seed, 1, 4, 4, 64, [128], trees, rng=rng)


def config2(B: int = 1) -> Workload:
    """Llama-3-8B-shaped layer: Hq=32, Hkv=8, D=128, L=2048, T=60 (expand+prune tree).
    B=1 is the configuration; B>1 repeats the shape with independent trees and
    values (the "same shape at saturating batch" extra)."""
    seed = BASE_SEED + 2
    rng = np.random.Generator(np.random.PCG64(seed))
    trees = [tree_expand_prune(rng, 60, 6, 4) for _ in range(B)]
    return make_workload("cfg2_8b" if B == 1 else f"cfg2_8b_B{B}", seed, B, 32, 8, 128,
                         [2048] * B, trees, rng=rng)


def config3(B: int) -> Workload:
    """Batch/cost sweep: Hq=32, Hkv=8, D=128, L_b ~ U{512..2048}, T = SWEEP[B], depth <= 8."""
    seed = BASE_SEED + 3 + 100 * B
    rng = np.random.Generator(np.random.PCG64(seed))
    L = rng.integers(512, 2049, size=B)
    trees = [tree_uniform(rng, SWEEP[B], 8) for _ in range(B)]
    return make_workload(f"cfg3_sweep_B{B}", seed, B, 32, 8, 128, L, trees, rng=rng)


def config4() -> Workload:
    """70B-shaped layer: B=8, Hq=64, Hkv=8, D=128, L=4096, T=32, depth <= 6."""
    seed = BASE_SEED + 4
    rng = np.random.Generator(np.random.PCG64(seed))
    trees = [tree_uniform(rng, 32, 6) for _ in range(8)]
    return make_workload("cfg4_70b", seed, 8, 64, 8, 128, [4096] * 8, trees, rng=rng)


def config5(l_lo: int = 16384, l_hi: int = 32768, B: int = 4) -> Workload:
    """Long-context paged KV: B=4, Hq=32, Hkv=8, D=128, L_b ~ U{16384..32768},
    16-token pages, seeded random page table over a shared pool, T=48, depth <= 7."""
    seed = BASE_SEED + 5
    rng = np.random.Generator(np.random.PCG64(seed))
    L = rng.integers(l_lo, l_hi + 1, size=B)
    trees = [tree_uniform(rng, 48, 7) for _ in range(B)]
    return make_workload("cfg5_paged", seed, B, 32, 8, 128, L, trees, page_size=16, rng=rng)


def random_workload(seed: int, B: int, Hq: int, Hkv: int, D: int, L, T, max_depth: int = 8,
                    page_size: int = 0, name: str = "random") -> Workload:
    """Small free-form workload for property tests: explicit per-sequence L and T."""
    rng = np.random.Generator(np.random.PCG64(seed))
    L = np.broadcast_to(np.asarray(L, dtype=np.int64), (B,))
    T = np.broadcast_to(np.asarray(T, dtype=np.int64), (B,))
    trees = [tree_uniform(rng, int(t), max_depth) if t > 0 else np.zeros(0, np.int32) for t in T]
    return make_workload(name, seed, B, Hq, Hkv, D, L, trees, page_size=page_size, rng=rng)
