"""GPU parity of the draft-tree construction kernels (through the C ABI) against the CPU oracles on the same seeded
inputs: selections, orders and indices compared exactly; the one float32 addition per candidate bit for bit."""
import numpy as np
import pytest

from oracle import cast_oracle as co
from oracle import draft_oracle as do
from paper_2510_26577_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch_dev():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2510_26577_amd import binding
    binding.load_library()
    return torch


def say(msg):
    print(msg, flush=True)


def run_expand(torch, cu_N, score, logp, K, ld=None, offset=0):
    """ld: row stride of the device copy (elements); offset: elements the first row starts behind a 16-byte boundary."""
    from paper_2510_26577_amd import draft
    n, V = logp.shape
    ld = ld or V
    flat = torch.full((n * ld + offset + 4,), float("nan"), dtype=torch.float32, device="cuda")
    rows = flat[offset:offset + n * ld].view(n, ld)[:, :V]
    rows.copy_(torch.from_numpy(logp))
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    max_N = int(np.diff(cu_N).max()) if len(cu_N) > 1 else 0
    cs, cp, ct = draft.expand_layer(d(cu_N, np.int32), d(score, np.float32), rows, K, max_N)
    torch.cuda.synchronize()
    return cs.cpu().numpy(), cp.cpu().numpy(), ct.cpu().numpy()


def check_expand(torch, cu_N, score, logp, K, **kw):
    ref = do.expand_layer(score, cu_N, logp, K)
    cs, cp, ct = run_expand(torch, cu_N, score, logp, K, **kw)
    for b, (rs, rp, rt) in enumerate(ref):
        o0, o1 = int(cu_N[b]) * K, int(cu_N[b + 1]) * K
        assert np.array_equal(cs[o0:o1], rs), b          # (== on floats: -0.0 equals 0.0, -inf equals -inf)
        assert np.array_equal(cp[o0:o1], rp) and np.array_equal(ct[o0:o1], rt), b


@pytest.mark.parametrize("n_rows,V,K,levels", [
    ([12], 32000, 12, 0),                 # one sequence, the paper's K-sized layer, Llama 2 vocabulary: 4 pieces per row
    ([10, 0, 7], 128256, 10, 0),          # Llama 3 vocabulary: 16 pieces, the last one ragged; a sequence without rows
    ([5, 12, 1, 8, 12, 3, 9, 2], 4099, 8, 0),   # V % 4 != 0: one token per load
    ([64, 40], 1000, 16, 0),              # 1024 candidates in one sequence: the whole sort
    ([5], 2 * 8192 + 5, 8, 0),            # a last piece with fewer tokens than K
    ([3], 7, 7, 0),                       # K = V
    ([6, 6], 50000, 12, 9),               # a handful of distinct log-probabilities per row: the tie rules decide
    ([4], 9000, 1, 3),                    # K = 1 with ties: the first of the equal maxima
    ([2], 262144, 16, 0),                 # 32 pieces x 16: the most one wave merges per row
])
def test_expand_layer_matches_oracle(torch_dev, n_rows, V, K, levels):
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(600 + V + K))
    cu_N, score, logp = wl.expansion_inputs(rng, n_rows, V, levels=levels)
    say(f"[case] expand n={n_rows} V={V} K={K} levels={levels}")
    check_expand(torch, cu_N, score, logp, K)


@pytest.mark.parametrize("B,n,V,K", [(1, 12, 50000, 12),     # one sequence, several pieces a row: the count rides in the last launch
                                      (1, 16, 128256, 16),    # the most that form takes: 256 candidates
                                      (1, 12, 8000, 12),      # one piece a row: the count is a launch of its own
                                      (1, 20, 20000, 8),      # more than 16 rows: the general path
                                      (4, 12, 32000, 12), (64, 3, 9000, 5)])
def test_expand_layer_with_the_breadth_decision(torch_dev, B, n, V, K):
    """tva_expand_layer asked for the breadth decision too: the candidates are the oracle's as without it, and the
    count, utility and cost are the oracle's breadth decision (Eq. 1, Eq. 2, Algorithm 1) on the candidates' values
    exp(score), for thresholds from "keep all" to "keep one"."""
    torch = torch_dev
    from paper_2510_26577_amd import draft
    rng = np.random.Generator(np.random.PCG64(4200 + B + n + V))
    cu_N, score, logp = wl.expansion_inputs(rng, [n] * B, V)
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    N = n * K
    M_rows, L, ctx = 4, 128, 200
    S_T = np.cumsum(rng.uniform(0.05, 0.3, (M_rows, N + 1)), axis=1) + 8.0
    S_D = np.cumsum(rng.uniform(0.002, 0.05, (M_rows, N + 1)), axis=1) + 0.5
    row = co.select_context(ctx, L, M_rows) // L - 1
    ref = do.expand_layer(score, cu_N, logp, K)
    values = np.stack([np.exp(r[0].astype(np.float64)).astype(np.float32) for r in ref])      # [B, N], descending
    say(f"[case] expand with the breadth decision B={B} n={n} V={V} K={K}")
    e_in = (d(cu_N, np.int32), d(score, np.float32), d(logp, np.float32), d(S_D[row, :N], np.float64))
    cs = torch.empty(B * N, dtype=torch.float32, device="cuda")
    cp = torch.empty(B * N, dtype=torch.int32, device="cuda")
    ct = torch.empty(B * N, dtype=torch.int32, device="cuda")
    need = draft.expand_workspace_bytes(B, V, K, B * n)
    ws = torch.empty(max(1, need // 8), dtype=torch.int64, device="cuda")
    count = torch.zeros(1, dtype=torch.int32, device="cuda")
    at = torch.zeros(2, dtype=torch.float64, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    counts = set()
    scale = float(values[:, 0].mean()) / float(S_D[row, 0] / S_T[row, 0])                     # the first candidate's slope
    for C1 in (-1e30, 0.0, 1e-4 * scale, 1e-2 * scale, 0.1 * scale, scale, 1e30):
        want, wu, wc = co.breadth_prune(values.tolist(), S_D.tolist(), S_T.tolist(), ctx, L, M_rows, C1)
        args = draft.make_expand_args(cu_N=e_in[0], score=e_in[1], logp=e_in[2], K=K, sum_N=B * n, max_N=n, cand_score=cs,
                                      cand_parent=cp, cand_token=ct, workspace=ws, workspace_bytes=need, draft_cost_row=e_in[3],
                                      target_cost_one=float(S_T[row, 0]), C1=C1, count=count, u_c_at=at, count_err_flag=flag)
        count.fill_(-1)
        draft.expand_layer_raw(args)
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        assert int(count.item()) == want, C1
        u_at, c_at = at.cpu().tolist()
        assert abs(u_at - wu) <= 1e-12 * max(1.0, abs(wu)) and abs(c_at - wc) <= 1e-15 * abs(wc), C1
        counts.add(want)
    assert len(counts) >= 3
    for b, (rs, rp, rt) in enumerate(ref):
        assert np.array_equal(cs.cpu().numpy()[b * N:(b + 1) * N], rs) and np.array_equal(ct.cpu().numpy()[b * N:(b + 1) * N], rt)
    # refused: sequences of different sizes, no cost row
    from paper_2510_26577_amd import binding
    if B > 1:
        bad = draft.make_expand_args(cu_N=e_in[0], score=e_in[1], logp=e_in[2], K=K, sum_N=B * n - 1, max_N=n, cand_score=cs,
                                     cand_parent=cp, cand_token=ct, workspace=ws, workspace_bytes=need, draft_cost_row=e_in[3],
                                     target_cost_one=1.0, C1=1.0, count=count)
        with pytest.raises(binding.TvaError):
            draft.expand_layer_raw(bad)
    bad = draft.make_expand_args(cu_N=e_in[0], score=e_in[1], logp=e_in[2], K=K, sum_N=B * n, max_N=n, cand_score=cs,
                                 cand_parent=cp, cand_token=ct, workspace=ws, workspace_bytes=need, target_cost_one=1.0, C1=1.0,
                                 count=count)
    with pytest.raises(binding.TvaError):
        draft.expand_layer_raw(bad)


def test_expand_layer_layouts_and_special_values(torch_dev):
    """Rows further apart than V, rows that do not start on 16 bytes (the one-token-per-load path on a vocabulary that
    would allow four), log-probabilities of -inf (tokens of probability zero; a row with fewer finite entries than K
    fills up with them, lowest token first) and of -0.0 next to 0.0."""
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(61))
    cu_N, score, logp = wl.expansion_inputs(rng, [7, 5], 20000, levels=0)
    say("[case] expand strides and offsets")
    check_expand(torch, cu_N, score, logp, 9, ld=20480)
    check_expand(torch, cu_N, score, logp, 9, ld=20001)
    check_expand(torch, cu_N, score, logp, 9, offset=1)
    say("[case] expand -inf and signed zeros")
    logp2 = logp.copy()
    logp2[:, 5000:] = -np.inf
    logp2[0, 3:] = -np.inf                             # three finite entries, K = 9
    logp2[1, :] = -np.inf
    logp2[1, 17] = 0.0                                 # a point mass
    logp2[2, [11, 4000]] = [-0.0, 0.0]                 # equal as numbers: token 11 first
    score2 = score.copy()
    score2[3] = -np.inf                                # a node of value zero: all its children too
    check_expand(torch, cu_N, score2, logp2, 9)


def test_expand_layer_when_few_threads_hold_the_large_values(torch_dev):
    """The selection bound (K-th largest of the per-thread maxima) lets more than 64 tokens through when three threads
    of a piece hold all its large values; the kernel then searches the maximum K times instead."""
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(62))
    V, K = 3 * 8192, 4
    cu_N, score, logp = wl.expansion_inputs(rng, [3], V)
    logp = np.minimum(logp, np.float32(-20.0))
    for t in range(3):                                  # thread t of a piece holds tokens 1024 i + 4 t + e
        for piece in range(3):
            idx = piece * 8192 + np.add.outer(1024 * np.arange(8), 4 * t + np.arange(4)).ravel()
            logp[:, idx] = (-1.0 - rng.random((3, 32))).astype(np.float32)
    say("[case] expand, large values held by three threads per piece")
    check_expand(torch, cu_N, score, logp, K)


def random_scored_tree(rng, M, ties=0.2):
    parent = np.array([-1] + [int(rng.integers(max(0, i - 9), i)) for i in range(1, M)], np.int32)
    score = np.zeros(M, np.float32)
    for i in range(1, M):
        score[i] = score[parent[i]] - (0.0 if rng.random() < ties else np.float32(rng.exponential(0.7)))
    return parent, score


def run_subtree(torch, score, parent, cu_M, cu_T, with_flag=True):
    from paper_2510_26577_amd import draft
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    flag = torch.zeros(1, dtype=torch.int32, device="cuda") if with_flag else None
    max_M = int(np.diff(cu_M).max())
    old, newp = draft.select_subtree(d(score, np.float32), d(parent, np.int32), d(cu_M, np.int32), d(cu_T, np.int32), max_M,
                                     err_flag=flag, total_kept=int(cu_T[-1]))
    torch.cuda.synchronize()
    return old.cpu().numpy(), newp.cpu().numpy(), (int(flag.item()) if with_flag else 0)


@pytest.mark.parametrize("sizes", [[1], [60], [300, 1, 17, 72], [2048, 5], [33] * 16])
def test_select_subtree_matches_oracle(torch_dev, sizes):
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(700 + len(sizes) + sizes[0]))
    trees = [random_scored_tree(rng, M) for M in sizes]
    cu_M = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([t[0] for t in trees])
    score = np.concatenate([t[1] for t in trees])
    say(f"[case] select_subtree sizes={sizes}")
    for pick in ("some", "all", "one", "none"):
        keep = [{"some": int(rng.integers(1, M + 1)), "all": M, "one": 1, "none": 0}[pick] for M in sizes]
        cu_T = np.concatenate([[0], np.cumsum(keep)]).astype(np.int32)
        old, newp, flag = run_subtree(torch, score, parent, cu_M, cu_T)
        assert flag == 0
        for b, (par, sc) in enumerate(trees):
            if keep[b] == 0:
                continue
            ro, rp = co.select_subtree(sc, par, keep[b])
            assert list(old[cu_T[b]:cu_T[b + 1]]) == ro and list(newp[cu_T[b]:cu_T[b + 1]]) == rp, (pick, b)


def test_select_subtree_flags_what_is_not_a_tree_of_the_method(torch_dev):
    torch = torch_dev
    parent = np.array([-1, 0, 1, -1, 0, 0], np.int32)
    score = np.array([0.0, -2.0, -1.0, 0.0, -1.0, -3.0], np.float32)     # node 2 scores above its parent 1
    cu_M = np.array([0, 3, 6], np.int32)
    with pytest.raises(ValueError):
        co.select_subtree(score[:3], parent[:3], 2)
    old, newp, flag = run_subtree(torch, score, parent, cu_M, np.array([0, 2, 4], np.int32))
    assert flag == 1                                                    # sequence 0
    assert list(old[2:4]) == [0, 1] and list(newp[2:4]) == [-1, 0]       # sequence 1 is untouched by it
    old, newp, flag = run_subtree(torch, score, parent, cu_M, np.array([0, 1, 5], np.int32))
    assert flag == 2                                                    # asked to keep 4 of 3 nodes
    assert list(old[:1]) == [0] and list(newp[:1]) == [-1]
    old, newp, _ = run_subtree(torch, score, parent, cu_M, np.array([0, 1, 3], np.int32), with_flag=False)
    assert list(old) == [0, 0, 1] and list(newp) == [-1, -1, 0]


@pytest.mark.parametrize("B,N_tot,m", [(1, 145, 72), (8, 145, 72), (64, 145, 72), (64, 160, 64), (3, 5, 72), (7, 37, 1),
                                        (5, 1, 4), (16, 300, 40), (2, 2048, 600)])
def test_rerank_count_matches_oracle(torch_dev, B, N_tot, m):
    """The number of nodes the cut keeps (Dynamic Reranking Stage) equals the oracle's for thresholds from one that
    keeps everything to one that keeps a single node, on trees whose scores come in any order and with ties; the
    prefix array it writes is what the cut takes; a cost row that does not increase is flagged."""
    torch = torch_dev
    from paper_2510_26577_amd import draft
    rng = np.random.Generator(np.random.PCG64(4000 + B + N_tot + m))
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    M_rows, L, n0 = 6, 256, 700
    N = min(N_tot, m)
    S_T = np.cumsum(rng.uniform(0.01, 0.3, (M_rows, max(N, 2))), axis=1) + 5.0 + np.arange(M_rows)[:, None]
    row = co.select_context(n0, L, M_rows) // L - 1
    # scores as the method makes them: log-values, a node's never above its parent's, in index (not score) order
    scores = np.empty((B, N_tot), np.float32)
    for j in range(B):
        par, sc = random_scored_tree(rng, N_tot)
        scores[j] = sc
    if N_tot > 4:
        scores[0, 3] = scores[0, 1]                                      # ties
    say(f"[case] rerank_count B={B} N_tot={N_tot} m={m}")
    counts = set()
    for C3 in (-1e30, 0.0, 1.0, 10.0, 30.0, 100.0, 300.0, 1000.0, 1e30):
        # (scores are logs, so utilities fall with the count: the thresholds are taken on the negated scale too)
        for sign in (1.0, -1.0):
            x = (sign * scores).astype(np.float32)
            want = co.rerank_count(x.tolist(), S_T.tolist(), n0, L, M_rows, m, C3)
            flag = torch.zeros(1, dtype=torch.int32, device="cuda")
            count, cu_T = draft.rerank_count(d(x, np.float32), d(S_T[row], np.float64), m, C3, err_flag=flag)
            torch.cuda.synchronize()
            assert int(flag.item()) == 0
            assert int(count.item()) == want, (C3, sign)
            assert cu_T.cpu().tolist() == [b * want for b in range(B + 1)]
            counts.add(want)
    if N > 3:
        assert len(counts) >= 2 + (N <= 100)                             # (the thresholds do move the count)
    bad = S_T[row].copy()
    if N >= 2:
        bad[N - 1] = bad[N - 2]
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        count, cu_T = draft.rerank_count(d(scores, np.float32), d(bad, np.float64), m, 0.1, err_flag=flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1 and int(count.item()) == 0 and not any(cu_T.cpu().tolist())


@pytest.mark.parametrize("B,N", [(1, 144), (8, 144), (64, 144), (3, 1), (5, 12), (2, 1024)])
def test_layer_breadth_count_matches_oracle_and_host(torch_dev, B, N):
    """The number of candidates a layer keeps (Eq. 1, Eq. 2, Algorithm 1 with C1): the count equals the oracle's, and
    count, utility and cost at the count equal the host routine's bit for bit (same additions in the same order), for
    thresholds from "keep all" to "keep one"; a cost row that does not increase is flagged."""
    torch = torch_dev
    from paper_2510_26577_amd import cast, draft
    rng = np.random.Generator(np.random.PCG64(4100 + B + N))
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    M_rows, L, ctx = 5, 128, 300
    S_T = np.cumsum(rng.uniform(0.05, 0.3, (M_rows, N + 1)), axis=1) + 8.0
    S_D = np.cumsum(rng.uniform(0.002, 0.05, (M_rows, N + 1)), axis=1) + 0.5
    row = co.select_context(ctx, L, M_rows) // L - 1
    # candidates' values in descending order per sample (probabilities: utilities grow with the count, ever more slowly)
    scores = -np.sort(-np.exp(-rng.exponential(2.0, (B, N))).astype(np.float32), axis=1)
    if N > 3:
        scores[0, 2] = scores[0, 1]
    say(f"[case] breadth_count B={B} N={N}")
    counts = set()
    for C1 in (-1e30, 0.0, 0.3, 1.0, 3.0, 10.0, 30.0, 1e30):
        hn, hu, hc = cast.breadth_prune(scores, S_D, S_T, ctx, L, C1)
        # (the oracle's double sums are quadratic in N: the largest case is checked against the host routine only,
        # which tests/test_cast_parity.py holds to the oracle)
        want, wu, wc = co.breadth_prune(scores.tolist(), S_D.tolist(), S_T.tolist(), ctx, L, M_rows, C1) if N <= 200 else (hn, hu, hc)
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        count, at = draft.breadth_count(d(scores, np.float32), d(S_D[row, :N], np.float64), float(S_T[row, 0]), C1, err_flag=flag)
        torch.cuda.synchronize()
        u_at, c_at = at.cpu().tolist()
        assert int(flag.item()) == 0
        assert int(count.item()) == want == hn, C1
        assert (u_at, c_at) == (hu, hc), C1
        assert abs(u_at - wu) <= 1e-12 * max(1.0, abs(wu)) and abs(c_at - wc) <= 1e-15 * abs(wc)
        counts.add(want)
    if 3 < N <= 200:
        assert len(counts) >= 3
    if N >= 2:
        bad = S_D[row, :N].copy()
        bad[N - 1] = bad[N - 2]
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        count, at = draft.breadth_count(d(scores, np.float32), d(bad, np.float64), float(S_T[row, 0]), 1.0, err_flag=flag)
        torch.cuda.synchronize()
        assert int(flag.item()) == 1 and int(count.item()) == 0


def test_rerank_count_refuses_what_does_not_fit(torch_dev):
    torch = torch_dev
    from paper_2510_26577_amd import binding, draft
    x = torch.zeros((2, 3000), dtype=torch.float32, device="cuda")
    cost = torch.arange(1, 3001, dtype=torch.float64, device="cuda")
    with pytest.raises(binding.TvaError):
        draft.rerank_count(x, cost, 72, 0.1)                             # a tree larger than the kernels rank
    with pytest.raises(binding.TvaError):
        draft.rerank_count(x[:, :1500].contiguous(), cost, 1500, 0.1)    # more ranks than the kernels weigh
    with pytest.raises(binding.TvaError):
        draft.rerank_count(x[:, :10].contiguous(), cost, 0, 0.1)
    with pytest.raises(binding.TvaError):
        draft.rerank_count(x[:, :10].contiguous(), cost, 5, 0.1, workspace=torch.empty(9, dtype=torch.float32, device="cuda"))


def test_a_tree_grown_and_cut_on_the_gpu_is_the_oracles_and_feeds_the_attention(torch_dev):
    """Four layers of expansion (the best 6 candidates of a layer are the next layer's rows, 4 children each), the cut to
    the 20 best nodes, and the ancestor masks of the result: the device path and the oracle path, run side by side on the
    same log-probabilities, grow the same tree, and the parents that come out are what tva_build_ancestor_mask takes."""
    torch = torch_dev
    from paper_2510_26577_amd import binding, draft
    rng = np.random.Generator(np.random.PCG64(63))
    B, V, K, width, depth, m = 3, 20000, 4, 6, 4, 20
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    # per sequence: nodes as (parent, token, score), root first; the current layer's node ids
    nodes = [[(-1, 0, np.float32(0.0))] for _ in range(B)]
    layer = [[0] for _ in range(B)]
    say("[case] grow, cut, mask")
    for _ in range(depth):
        n_rows = [len(l) for l in layer]
        cu_N, _, logp = wl.expansion_inputs(rng, n_rows, V)
        score = np.array([nodes[b][i][2] for b in range(B) for i in layer[b]], np.float32)
        ref = do.expand_layer(score, cu_N, logp, K)
        cs, cp, ct = draft.expand_layer(d(cu_N, np.int32), d(score, np.float32), d(logp, np.float32), K, max(n_rows))
        torch.cuda.synchronize()
        cs, cp, ct = cs.cpu().numpy(), cp.cpu().numpy(), ct.cpu().numpy()
        for b in range(B):
            o0 = int(cu_N[b]) * K
            rs, rp, rt = ref[b]
            take = min(width, len(rs))
            assert np.array_equal(cs[o0:o0 + take], rs[:take]) and np.array_equal(cp[o0:o0 + take], rp[:take])
            assert np.array_equal(ct[o0:o0 + take], rt[:take])
            nxt = []
            for j in range(take):
                nodes[b].append((layer[b][int(cp[o0 + j])], int(ct[o0 + j]), np.float32(cs[o0 + j])))
                nxt.append(len(nodes[b]) - 1)
            layer[b] = nxt
    sizes = [len(x) for x in nodes]
    cu_M = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    cu_T = (np.arange(B + 1) * m).astype(np.int32)
    parent = np.array([x[0] for seq in nodes for x in seq], np.int32)
    score = np.array([x[2] for seq in nodes for x in seq], np.float32)
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    old, newp = draft.select_subtree(d(score, np.float32), d(parent, np.int32), d(cu_M, np.int32), d(cu_T, np.int32), max(sizes),
                                     err_flag=flag, total_kept=B * m)
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    old, newp = old.cpu().numpy(), newp.cpu().numpy()
    for b in range(B):
        ro, rp = co.select_subtree(score[cu_M[b]:cu_M[b + 1]], parent[cu_M[b]:cu_M[b + 1]], m)
        assert list(old[b * m:(b + 1) * m]) == ro and list(newp[b * m:(b + 1) * m]) == rp
    mask, status, bad = binding.build_ancestor_mask_host(newp, cu_T, m)
    assert status == 0 and bad == -1                                   # a tree in topological order
    assert all(int(mask[b * m, 0]) == 1 for b in range(B))             # node 0 of every tree is its own only ancestor


@pytest.mark.parametrize("node_count", [False, True])
def test_draft_and_sampling_kernels_replayed_from_a_graph(torch_dev, node_count):
    """tva_expand_layer, tva_tree_select_subtree and tva_accept_sampling (several workgroups per sequence: a
    counter-zeroing kernel -- with the host's node count the kernel that sums the rows ahead of the walk -- then the
    walk with its waits) captured in one HIP graph: every replay, with the outputs and the scratch memory overwritten
    by eager work in between, reproduces the eager results bit for bit."""
    torch = torch_dev
    from paper_2510_26577_amd import draft, verify
    from oracle import verify_oracle as vo
    rng = np.random.Generator(np.random.PCG64(64))
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    # expansion
    K, V = 8, 50000
    cu_N, score, logp = wl.expansion_inputs(rng, [9, 4, 12], V)
    n_rows = int(cu_N[-1])
    cs = torch.empty(n_rows * K, dtype=torch.float32, device="cuda")
    cp = torch.empty(n_rows * K, dtype=torch.int32, device="cuda")
    ct = torch.empty(n_rows * K, dtype=torch.int32, device="cuda")
    need = draft.expand_workspace_bytes(3, V, K, n_rows)
    ws = torch.empty(need // 8, dtype=torch.int64, device="cuda")
    e_in = (d(cu_N, np.int32), d(score, np.float32), d(logp, np.float32))     # (kept alive: the argument block holds pointers)
    eargs = draft.make_expand_args(cu_N=e_in[0], score=e_in[1], logp=e_in[2], K=K, sum_N=n_rows,
                                   max_N=12, cand_score=cs, cand_parent=cp, cand_token=ct, workspace=ws, workspace_bytes=need)
    # subtree cut
    sizes, m = [90, 40], 25
    trees = [random_scored_tree(rng, M) for M in sizes]
    cu_M = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    cu_T = (np.arange(len(sizes) + 1) * m).astype(np.int32)
    t_score, t_parent = d(np.concatenate([t[1] for t in trees]), np.float32), d(np.concatenate([t[0] for t in trees]), np.int32)
    d_cu_M, d_cu_T = d(cu_M, np.int32), d(cu_T, np.int32)
    old = torch.empty(len(sizes) * m, dtype=torch.int32, device="cuda")
    newp = torch.empty(len(sizes) * m, dtype=torch.int32, device="cuda")
    # sampling
    Vs, T = 60000, np.array([14, 9])
    s_cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    s_parent = np.concatenate([wl.tree_expand_prune(rng, int(t)) for t in T]).astype(np.int32)
    p, q, tok, u, uf = wl.sampling_inputs(rng, s_parent, s_cu_T, Vs, drift=0.4)
    sargs = (d(s_parent, np.int32), d(s_cu_T, np.int32), d(tok, np.int32), d(p, np.float32), d(q, np.float32), d(u, np.float32),
             d(uf, np.float32), 6)
    residual = torch.empty((2, Vs), dtype=torch.float32, device="cuda")
    sum_T = int(s_cu_T[-1]) if node_count else 0
    sws = torch.empty(verify._lib().tva_sample_workspace_bytes_rows(2, sum_T, Vs) // 8, dtype=torch.int64, device="cuda")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    results = {}
    # the count of nodes to keep (trees of equal size: the first 40 scores of each)
    r_scores = torch.stack([t_score[:40], t_score[90:130]]).contiguous()
    r_cost = torch.cumsum(torch.full((25,), 0.03, dtype=torch.float64, device="cuda"), 0) + 4.0
    r_count = torch.zeros(1, dtype=torch.int32, device="cuda")
    r_cu = torch.zeros(3, dtype=torch.int32, device="cuda")
    r_ws = torch.empty(2 * 25, dtype=torch.float32, device="cuda")

    def one_pass(stream=None):
        draft.rerank_count(r_scores, r_cost, 25, -40.0, count=r_count, cu_T=r_cu, err_flag=flag, stream=stream, workspace=r_ws)
        draft.expand_layer_raw(eargs, stream)
        draft.select_subtree(t_score, t_parent, d_cu_M, d_cu_T, max(sizes), old_index=old, new_parent=newp, err_flag=flag, stream=stream)
        results["path"], results["n"], results["next"] = verify.accept_sampling(
            *sargs, residual=residual, err_flag=flag, stream=stream, workspace=sws, workgroups_per_sequence=8, sum_T=sum_T)

    say("[case] draft + sampling kernels, eager")
    one_pass()
    torch.cuda.synchronize()
    assert int(flag.item()) == 0
    ref_paths, ref_next = vo.accept_sampling(s_parent, s_cu_T, tok, p, q, u, uf, max_path=6)
    assert results["next"].cpu().tolist() == ref_next and results["n"].cpu().tolist() == [len(x) for x in ref_paths]
    ref = do.expand_layer(score, cu_N, logp, K)
    assert np.array_equal(cs.cpu().numpy()[:9 * K], ref[0][0]) and np.array_equal(ct.cpu().numpy()[:9 * K], ref[0][2])
    want_count = co.rerank_count(r_scores.cpu().tolist(), [r_cost.cpu().tolist()], 0, 256, 1, 25, -40.0)
    assert int(r_count.item()) == want_count and r_cu.cpu().tolist() == [0, want_count, 2 * want_count]
    eager = [t.clone() for t in (cs, cp, ct, old, newp, results["path"], results["n"], results["next"], r_count, r_cu)]

    def scribble():
        for t in (cs, residual):
            t.fill_(float("nan"))
        for t in (cp, ct, old, newp, ws, sws, r_count, r_cu):
            t.fill_(-7)
        r_ws.fill_(float("nan"))
        flag.zero_()

    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    scribble()
    torch.cuda.synchronize()
    with torch.cuda.graph(g, stream=side):
        one_pass(side)
    graph_outs = (cs, cp, ct, old, newp, results["path"], results["n"], results["next"], r_count, r_cu)
    for replay in range(3):
        say(f"[case] draft + sampling kernels, graph replay {replay}")
        scribble()                                # eager work between the replays
        for t in graph_outs[5:8]:
            t.fill_(-9)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(flag.item()) == 0
        for name, got, want in zip("cand_score cand_parent cand_token old_index new_parent path path_len next count cu_T".split(), graph_outs, eager):
            assert torch.equal(got, want), (name, replay)
