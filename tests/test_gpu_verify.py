"""GPU parity of tree acceptance (greedy, and by speculative sampling) and the K/V commit (through the C ABI)
against the CPU oracle on the same seeded inputs: integer and byte work, compared exactly."""
import numpy as np
import pytest

from oracle import verify_oracle as vo
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


def make_tokens(rng, parent, cu_T, vocab, plant):
    """Draft tokens with distinct siblings, target tokens random with `plant` of them set to a child's token."""
    sum_T = int(cu_T[-1])
    draft = np.zeros(sum_T, np.int32)
    target = rng.integers(0, vocab, sum_T).astype(np.int32)
    for b in range(len(cu_T) - 1):
        t0, T = int(cu_T[b]), int(cu_T[b + 1] - cu_T[b])
        used = {}
        kids = {}
        for i in range(T):
            p = int(parent[t0 + i])
            kids.setdefault(p, []).append(i)
            while True:
                t = int(rng.integers(0, vocab))
                if t not in used.setdefault(p, set()):
                    used[p].add(t)
                    draft[t0 + i] = t
                    break
        for i in range(T):
            if i in kids and rng.random() < plant:
                target[t0 + i] = draft[t0 + kids[i][int(rng.integers(0, len(kids[i])))]]
    return draft, target


def run_accept(torch, parent, cu_T, draft, target, max_path):
    from paper_2510_26577_amd import verify
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    path, n, nxt = verify.accept_greedy(d(parent), d(cu_T), d(draft), d(target), max_path)
    torch.cuda.synchronize()
    return path.cpu().numpy(), n.cpu().numpy(), nxt.cpu().numpy()


@pytest.mark.parametrize("B,T_hi,plant", [(1, 8, 0.9), (4, 60, 0.8), (64, 72, 0.7), (16, 300, 0.95), (7, 1, 0.5)])
def test_accept_greedy_matches_oracle(torch_dev, B, T_hi, plant):
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(31 + B + T_hi))
    T = rng.integers(0 if B > 4 else 1, T_hi + 1, B)
    T[0] = T_hi
    cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    parent = np.concatenate([wl.tree_uniform(rng, int(t), 40) if t > 0 else np.zeros(0, np.int32) for t in T]).astype(np.int32)
    draft, target = make_tokens(rng, parent, cu_T, vocab=100, plant=plant)
    say(f"[case] accept B={B} T<={T_hi} plant={plant}")
    for max_path in (int(T.max()) + 1, 3, 1):
        ref_paths, ref_next = vo.accept_greedy(parent, cu_T, draft, target, max_path=max_path)
        path, n, nxt = run_accept(torch, parent, cu_T, draft, target, max_path)
        assert list(n) == [len(p) for p in ref_paths]
        assert list(nxt) == ref_next
        for b, p in enumerate(ref_paths):
            assert list(path[b, :len(p)]) == p
    assert max(len(p) for p in vo.accept_greedy(parent, cu_T, draft, target)[0]) >= (3 if T_hi >= 8 else 1)


def test_accept_duplicate_sibling_tokens_take_the_lowest_index(torch_dev):
    torch = torch_dev
    parent = np.array([-1, 0, 0, 0, 2, 2], np.int32)
    draft = np.array([0, 5, 5, 5, 9, 9], np.int32)
    target = np.array([5, 1, 9, 1, 1, 1], np.int32)      # root -> first child with token 5 = node 1, which has no children
    path, n, nxt = run_accept(torch, parent, np.array([0, 6], np.int32), draft, target, 6)
    assert list(path[0, :n[0]]) == [0, 1] and nxt[0] == 1
    draft[1] = 4                                          # now node 2 is the first match, then node 4
    path, n, nxt = run_accept(torch, parent, np.array([0, 6], np.int32), draft, target, 6)
    assert list(path[0, :n[0]]) == [0, 2, 4] and nxt[0] == 1


def _commit_case(torch, w, paths, paged_capacity_tokens=None, strides_head_major=False):
    """Runs the commit on the GPU for workload w (dense or paged) and returns what the oracle needs to compare."""
    from paper_2510_26577_amd import verify
    B = w.B
    max_path = max(1, max(len(p) for p in paths))
    path = np.full((B, max_path), -1, np.int32)
    for b, p in enumerate(paths):
        path[b, :len(p)] = p
    plen = np.array([len(p) for p in paths], np.int32)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    as_i16 = lambda a: a.view(np.int16)
    return verify, dev, as_i16, path, plen


@pytest.mark.parametrize("B,Hkv,D", [(3, 2, 64), (8, 8, 128), (64, 8, 128)])
def test_commit_dense_matches_oracle(torch_dev, B, Hkv, D):
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(41 + B))
    T = rng.integers(1, 40, B)
    L = rng.integers(0, 300, B).astype(np.int32)
    w = wl.random_workload(900 + B, B, Hkv * 2, Hkv, D, L, T)
    # capacity: room for a few more tokens per sequence; sequence 0 gets too little on purpose
    cap = L + rng.integers(6, 20, B)
    paths = []
    for b in range(B):
        n = int(rng.integers(1, min(int(T[b]), 6) + 1))
        paths.append(sorted(rng.choice(int(T[b]), size=n, replace=False).tolist()))
    cu_cap = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
    kc = rng.integers(0, 2 ** 16, (int(cap.sum()), Hkv, D)).astype(np.uint16)
    vc = rng.integers(0, 2 ** 16, (int(cap.sum()), Hkv, D)).astype(np.uint16)
    verify, dev, as_i16, path, plen = _commit_case(torch, w, paths)
    say(f"[case] commit dense B={B} Hkv={Hkv} D={D}")
    k_d, v_d = dev(as_i16(kc)), dev(as_i16(vc))
    L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    verify.commit_path(cu_T=dev(w.cu_T), L=dev(L), path=dev(path), path_len=dev(plen), k_tree=dev(as_i16(w.k_tree)),
                       v_tree=dev(as_i16(w.v_tree)), k_cache=k_d, v_cache=v_d, cu_L=dev(cu_cap), L_out=L_out, err_flag=err)
    torch.cuda.synchronize()
    k_ref, v_ref, L_ref = vo.commit_path_dense(kc, vc, cu_cap, L, w.k_tree, w.v_tree, w.cu_T, paths)
    assert int(err.item()) == 0
    assert np.array_equal(k_d.cpu().numpy().view(np.uint16), k_ref) and np.array_equal(v_d.cpu().numpy().view(np.uint16), v_ref)
    assert np.array_equal(L_out.cpu().numpy(), L_ref)
    # no room: the flag names the sequence, rows inside the room are still written, nothing outside it is
    tight = cap.copy()
    tight[B - 1] = L[B - 1] + len(paths[B - 1]) - 1
    cu_tight = np.concatenate([[0], np.cumsum(tight)]).astype(np.int32)
    kc2 = rng.integers(0, 2 ** 16, (int(tight.sum()) + 1, Hkv, D)).astype(np.uint16)   # one guard row at the end
    k2, v2 = dev(as_i16(kc2)), dev(as_i16(kc2.copy()))
    err.zero_()
    verify.commit_path(cu_T=dev(w.cu_T), L=dev(L), path=dev(path), path_len=dev(plen), k_tree=dev(as_i16(w.k_tree)),
                       v_tree=dev(as_i16(w.v_tree)), k_cache=k2, v_cache=v2, cu_L=dev(cu_tight), err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == B
    assert np.array_equal(k2.cpu().numpy().view(np.uint16)[-1], kc2[-1])


@pytest.mark.parametrize("page_size", [16, 1, 5])
def test_commit_paged_matches_oracle(torch_dev, page_size):
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(51 + page_size))
    B, Hkv, D = 6, 4, 128
    T = rng.integers(1, 30, B)
    L = rng.integers(0, 100, B).astype(np.int32)
    w = wl.random_workload(950 + page_size, B, Hkv, Hkv, D, L, T)
    paths = [sorted(rng.choice(int(T[b]), size=int(rng.integers(1, min(int(T[b]), 8) + 1)), replace=False).tolist()) for b in range(B)]
    max_pages = int((L.max() + 8 + page_size - 1) // page_size) + 1
    perm = rng.permutation(B * max_pages).reshape(B, max_pages).astype(np.int32)
    kp = rng.integers(0, 2 ** 16, (B * max_pages, page_size, Hkv, D)).astype(np.uint16)
    vp = rng.integers(0, 2 ** 16, (B * max_pages, page_size, Hkv, D)).astype(np.uint16)
    verify, dev, as_i16, path, plen = _commit_case(torch, w, paths)
    say(f"[case] commit paged page_size={page_size}")
    k_d, v_d = dev(as_i16(kp)), dev(as_i16(vp))
    L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
    verify.commit_path(cu_T=dev(w.cu_T), L=dev(L), path=dev(path), path_len=dev(plen), k_tree=dev(as_i16(w.k_tree)),
                       v_tree=dev(as_i16(w.v_tree)), k_cache=k_d, v_cache=v_d, page_table=dev(perm), page_size=page_size,
                       L_out=L_out)
    torch.cuda.synchronize()
    k_ref, v_ref, L_ref = vo.commit_path_paged(kp, vp, perm, page_size, L, w.k_tree, w.v_tree, w.cu_T, paths)
    assert np.array_equal(k_d.cpu().numpy().view(np.uint16), k_ref) and np.array_equal(v_d.cpu().numpy().view(np.uint16), v_ref)
    assert np.array_equal(L_out.cpu().numpy(), L_ref)


@pytest.mark.parametrize("form", ["dense", "paged", "in place dense", "in place paged"])
def test_commit_of_all_layers_in_one_call(torch_dev, form):
    """n_layers > 1: the layers' caches (and tree tensors) lie layer_stride elements apart, with a gap of unrelated
    data between them; one call commits every layer as the oracle commits each of them, leaves the gaps alone, and
    writes L_out once."""
    torch = torch_dev
    from paper_2510_26577_amd import verify
    rng = np.random.Generator(np.random.PCG64(61 + len(form)))
    layers, B, Hkv, D, page_size = 5, 4, 2, 64, 4
    paged, in_place = "paged" in form, "in place" in form
    T = np.array([9, 1, 30, 17])
    L = np.array([20, 0, 7, 64], np.int32)
    ws = [wl.random_workload(1500 + l, B, Hkv, Hkv, D, L, T, max_depth=6) for l in range(layers)]   # one tree, K/V per layer
    parent = ws[0].parent
    draft, target = make_tokens(rng, parent, ws[0].cu_T, vocab=30, plant=0.9)
    paths, _ = vo.accept_greedy(parent, ws[0].cu_T, draft, target, max_path=8)
    max_path = 8
    path = np.full((B, max_path), -1, np.int32)
    for b, p_ in enumerate(paths):
        path[b, :len(p_)] = p_
    plen = np.array([len(p_) for p_ in paths], np.int32)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    cap = L + T + 3
    cu = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
    max_pages = int((cap.max() + page_size - 1) // page_size)
    table = rng.permutation(B * max_pages).reshape(B, max_pages).astype(np.int32)
    rows = B * max_pages * page_size if paged else int(cap.sum())
    gap = 24                                                     # elements of unrelated data between two layers' tensors
    per_layer = rows * Hkv * D
    def layered(fill):
        buf = rng.integers(0, 2 ** 16, layers * (per_layer + gap)).astype(np.uint16)
        for l in range(layers):
            buf[l * (per_layer + gap): l * (per_layer + gap) + per_layer] = fill(l).reshape(-1)
        return buf
    def pool(l, which):
        x = rng.integers(0, 2 ** 16, (rows, Hkv, D)).astype(np.uint16)
        if in_place:                                             # the tree's rows sit behind the committed ones
            src = ws[l].k_tree if which == "k" else ws[l].v_tree
            for b in range(B):
                for i in range(int(T[b])):
                    t = int(L[b]) + i
                    r = table[b, t // page_size] * page_size + t % page_size if paged else cu[b] + t
                    x[r] = src[ws[l].cu_T[b] + i]
        return x
    k0 = [pool(l, "k") for l in range(layers)]
    v0 = [pool(l, "v") for l in range(layers)]
    kbuf, vbuf = layered(lambda l: k0[l]), layered(lambda l: v0[l])
    tree_rows = int(T.sum()) * Hkv * D
    ktree = np.concatenate([np.concatenate([ws[l].k_tree.reshape(-1), rng.integers(0, 2 ** 16, gap).astype(np.uint16)]) for l in range(layers)])
    vtree = np.concatenate([np.concatenate([ws[l].v_tree.reshape(-1), rng.integers(0, 2 ** 16, gap).astype(np.uint16)]) for l in range(layers)])
    i16 = lambda a: a.view(np.int16)
    k_d, v_d = dev(i16(kbuf)), dev(i16(vbuf))
    first = lambda t: t[:per_layer].view((rows // page_size, page_size, Hkv, D) if paged else (rows, Hkv, D))
    kt_d, vt_d = dev(i16(ktree)), dev(i16(vtree))
    L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    say(f"[case] commit of {layers} layers in one call, {form}")
    verify.commit_path(cu_T=dev(ws[0].cu_T), L=dev(L), path=dev(path), path_len=dev(plen),
                       k_tree=None if in_place else kt_d[:tree_rows].view(int(T.sum()), Hkv, D),
                       v_tree=None if in_place else vt_d[:tree_rows].view(int(T.sum()), Hkv, D),
                       k_cache=first(k_d), v_cache=first(v_d), cu_L=None if paged else dev(cu),
                       page_table=dev(table) if paged else None, page_size=page_size if paged else 0, L_out=L_out, err_flag=err,
                       n_layers=layers, layer_stride_cache=per_layer + gap, layer_stride_tree=tree_rows + gap)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    assert np.array_equal(L_out.cpu().numpy(), L + plen)
    k_ref, v_ref = kbuf.copy(), vbuf.copy()
    for l in range(layers):
        if in_place:
            ek, ev = k0[l].copy(), v0[l].copy()
            for b, p_ in enumerate(paths):
                for j, node in enumerate(p_):
                    t_src, t_dst = int(L[b]) + node, int(L[b]) + j
                    rs = table[b, t_src // page_size] * page_size + t_src % page_size if paged else cu[b] + t_src
                    rd = table[b, t_dst // page_size] * page_size + t_dst % page_size if paged else cu[b] + t_dst
                    ek[rd], ev[rd] = k0[l][rs], v0[l][rs]
        elif paged:
            ek, ev, _ = vo.commit_path_paged(k0[l].reshape(-1, page_size, Hkv, D), v0[l].reshape(-1, page_size, Hkv, D), table, page_size,
                                             L, ws[l].k_tree, ws[l].v_tree, ws[l].cu_T, paths)
        else:
            ek, ev, _ = vo.commit_path_dense(k0[l], v0[l], cu, L, ws[l].k_tree, ws[l].v_tree, ws[l].cu_T, paths)
        o = l * (per_layer + gap)
        k_ref[o:o + per_layer], v_ref[o:o + per_layer] = ek.reshape(-1), ev.reshape(-1)
    assert np.array_equal(k_d.cpu().numpy().view(np.uint16), k_ref) and np.array_equal(v_d.cpu().numpy().view(np.uint16), v_ref)


def test_accept_then_commit_then_attend(torch_dev):
    """The committed rows are what the next step's attention reads: after commit, attention over the longer cache
    (with a one-node tree) equals the oracle on the host-side committed cache."""
    torch = torch_dev
    from oracle import tva_oracle as orc
    from paper_2510_26577_amd import device, verify
    rng = np.random.Generator(np.random.PCG64(61))
    B, Hq, Hkv, D = 3, 8, 2, 128
    L = np.array([40, 0, 129], np.int32)
    T = np.array([12, 5, 30])
    w = wl.random_workload(990, B, Hq, Hkv, D, L, T)
    draft, target = make_tokens(rng, w.parent, w.cu_T, vocab=30, plant=0.9)
    paths, _ = vo.accept_greedy(w.parent, w.cu_T, draft, target)
    cap = L + T
    cu_cap = np.concatenate([[0], np.cumsum(cap)]).astype(np.int32)
    kc = np.zeros((int(cap.sum()), Hkv, D), np.uint16)
    vc = np.zeros_like(kc)
    for b in range(B):
        kc[cu_cap[b]:cu_cap[b] + L[b]] = w.k_cache[w.cu_L[b]:w.cu_L[b] + L[b]]
        vc[cu_cap[b]:cu_cap[b] + L[b]] = w.v_cache[w.cu_L[b]:w.cu_L[b] + L[b]]
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    i16 = lambda a: a.view(np.int16)
    dp, dcu = dev(w.parent), dev(w.cu_T)
    path, plen, nxt = verify.accept_greedy(dp, dcu, dev(draft), dev(target), int(T.max()))
    k_d, v_d = dev(i16(kc)), dev(i16(vc))
    L_new = torch.zeros(B, dtype=torch.int32, device="cuda")
    verify.commit_path(cu_T=dcu, L=dev(L), path=path, path_len=plen, k_tree=dev(i16(w.k_tree)), v_tree=dev(i16(w.v_tree)),
                       k_cache=k_d, v_cache=v_d, cu_L=dev(cu_cap), L_out=L_new)
    torch.cuda.synchronize()
    assert [list(path[b, :plen[b]].cpu().numpy()) for b in range(B)] == paths
    k_ref, v_ref, L_ref = vo.commit_path_dense(kc, vc, cu_cap, L, w.k_tree, w.v_tree, w.cu_T, paths)
    assert np.array_equal(L_new.cpu().numpy(), L_ref)
    # next step: one new token per sequence attends to the committed cache
    import dataclasses
    w2 = wl.random_workload(991, B, Hq, Hkv, D, L_ref, [1] * B)
    w2 = dataclasses.replace(w2, k_cache=k_ref, v_cache=v_ref, cu_L=cu_cap)
    dw2 = device.to_device(w2)
    dw2.k_cache, dw2.v_cache = k_d, v_d                     # the GPU reads what the commit kernel wrote
    out, lse = device.attention(dw2, None)
    torch.cuda.synchronize()
    ro, rl = orc.tree_verify_attn(w2)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= 2e-3
    assert np.abs(lse.cpu().numpy().astype(np.float64) - rl).max() <= 1e-4


def _in_cache_layout(w, rng, page_size=0):
    """Re-stores a workload with its tree K/V appended to each sequence's cache: returns the host arrays
    (k, v, cu_L or page_table).  Position t < L_b is cached token t, position L_b + i is tree node i."""
    B, Hkv, D = w.B, w.Hkv, w.D
    tot = w.L.astype(np.int64) + w.T.astype(np.int64)

    def rows_of(b, cache, tree):
        if w.paged:
            src = np.stack([cache[w.page_table[b, t // w.page_size], t % w.page_size] for t in range(int(w.L[b]))]) \
                if w.L[b] else np.zeros((0, Hkv, D), np.uint16)
        else:
            src = cache[w.cu_L[b]:w.cu_L[b] + w.L[b]]
        return np.concatenate([src, tree[w.cu_T[b]:w.cu_T[b + 1]]])

    if page_size == 0:
        cu = np.concatenate([[0], np.cumsum(tot)]).astype(np.int32)
        k = np.concatenate([rows_of(b, w.k_cache, w.k_tree) for b in range(B)])
        v = np.concatenate([rows_of(b, w.v_cache, w.v_tree) for b in range(B)])
        return k, v, cu, None
    max_pages = int((tot.max() + page_size - 1) // page_size) + 1
    table = rng.permutation(B * max_pages).reshape(B, max_pages).astype(np.int32)
    k = rng.integers(0, 2 ** 16, (B * max_pages, page_size, Hkv, D)).astype(np.uint16) | np.uint16(0x7F80)  # NaN/inf filler
    v = k.copy()
    for b in range(B):
        kr, vr = rows_of(b, w.k_cache, w.k_tree), rows_of(b, w.v_cache, w.v_tree)
        for t in range(int(tot[b])):
            k[table[b, t // page_size], t % page_size] = kr[t]
            v[table[b, t // page_size], t % page_size] = vr[t]
    return k, v, None, table


@pytest.mark.parametrize("page_size", [0, 16, 3])
@pytest.mark.parametrize("variant", [0, 1, 3, 5])
def test_attention_with_tree_rows_in_the_cache(torch_dev, page_size, variant):
    """k_tree = v_tree = NULL: the kernel reads the tree tokens' K/V from cache positions L_b + i; the
    result must equal the oracle's on the same values held in separate tree tensors."""
    torch = torch_dev
    from oracle import tva_oracle as orc
    from paper_2510_26577_amd import binding
    rng = np.random.Generator(np.random.PCG64(71 + page_size))
    w = wl.random_workload(1000 + page_size, 4, 8, 2, 128, [300, 64, 0, 129], [70, 33, 8, 128], max_depth=12)
    k, v, cu, table = _in_cache_layout(w, rng, page_size)
    say(f"[case] in-cache tree rows, page_size={page_size} variant={variant}")
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    i16 = lambda a: a.view(np.int16)
    q, cu_T, L, parent = dev(i16(w.q)), dev(w.cu_T), dev(w.L.astype(np.int32)), dev(w.parent)
    for splits in (0, 3):
        out, lse = binding.tree_verify_attn(q, None, None, dev(i16(k)), dev(i16(v)), None, cu_T, L, max_T=w.max_T,
                                            max_L=w.max_L, scale=w.scale, cu_L=dev(cu), page_table=dev(table),
                                            page_size=page_size, num_splits=splits, parent=parent,
                                            plan_shape=variant)
        torch.cuda.synchronize()
        ro, rl = orc.tree_verify_attn(w)
        assert np.isfinite(out.cpu().numpy()).all()
        assert np.abs(out.cpu().numpy().astype(np.float64) - ro).max() <= 2e-3
        assert np.abs(lse.cpu().numpy().astype(np.float64) - rl).max() <= 1e-4 <= 1e-4


@pytest.mark.parametrize("page_size", [0, 16, 5])
def test_commit_in_place_for_tree_rows_in_the_cache(torch_dev, page_size):
    torch = torch_dev
    from paper_2510_26577_amd import verify
    rng = np.random.Generator(np.random.PCG64(81 + page_size))
    B = 5
    T = np.array([40, 1, 9, 72, 17])
    L = np.array([100, 0, 31, 5, 64], np.int32)
    w = wl.random_workload(1100 + page_size, B, 4, 4, 128, L, T, max_depth=13)
    k, v, cu, table = _in_cache_layout(w, rng, page_size)
    # deep trees (each parent among the two previous nodes) so that accepted paths get long
    deep = np.concatenate([np.array([-1] + [int(rng.integers(max(0, i - 2), i)) for i in range(1, int(t))], np.int32)
                           for t in T])
    draft, target = make_tokens(rng, deep, w.cu_T, vocab=40, plant=0.95)
    paths, _ = vo.accept_greedy(deep, w.cu_T, draft, target, max_path=16)
    assert max(len(p) for p in paths) >= 6 and any(p != list(range(len(p))) for p in paths)
    max_path = 16
    path = np.full((B, max_path), -1, np.int32)
    for b, p in enumerate(paths):
        path[b, :len(p)] = p
    plen = np.array([len(p) for p in paths], np.int32)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    i16 = lambda a: a.view(np.int16)
    k_d, v_d = dev(i16(k)), dev(i16(v))
    L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    say(f"[case] in-place commit, page_size={page_size}")
    verify.commit_path(cu_T=dev(w.cu_T), L=dev(L), path=dev(path), path_len=dev(plen), k_tree=None, v_tree=None,
                       k_cache=k_d, v_cache=v_d, cu_L=dev(cu), page_table=dev(table), page_size=page_size,
                       L_out=L_out, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    # expected: position L_b + j holds the old row of position L_b + path[j]; every other position is unchanged
    k_ref, v_ref = k.copy(), v.copy()

    def at(arr, b, t):
        return arr[cu[b] + t] if page_size == 0 else arr[table[b, t // page_size], t % page_size]

    for b, p in enumerate(paths):
        for j, node in enumerate(p):
            if page_size == 0:
                k_ref[cu[b] + L[b] + j], v_ref[cu[b] + L[b] + j] = at(k, b, L[b] + node), at(v, b, L[b] + node)
            else:
                t = L[b] + j
                k_ref[table[b, t // page_size], t % page_size] = at(k, b, L[b] + node)
                v_ref[table[b, t // page_size], t % page_size] = at(v, b, L[b] + node)
    assert np.array_equal(k_d.cpu().numpy().view(np.uint16), k_ref) and np.array_equal(v_d.cpu().numpy().view(np.uint16), v_ref)
    assert np.array_equal(L_out.cpu().numpy(), L + plen)
    # a row that is not a rising path is refused
    bad = path.copy()
    b_long = int(np.argmax(plen))
    bad[b_long, 1] = 0
    err.zero_()
    verify.commit_path(cu_T=dev(w.cu_T), L=dev(L), path=dev(bad), path_len=dev(plen), k_tree=None, v_tree=None,
                       k_cache=k_d, v_cache=v_d, cu_L=dev(cu), page_table=dev(table), page_size=page_size, err_flag=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 1 + b_long


@pytest.mark.parametrize("page_size", [0, 16])
def test_whole_pass_replayed_from_a_graph(torch_dev, page_size):
    """Attention on tree rows held in the cache, acceptance and in-place commit captured in one HIP graph:
    every replay (cache restored by eager work in between) must reproduce the eager pass bit for bit."""
    torch = torch_dev
    from paper_2510_26577_amd import binding, verify
    rng = np.random.Generator(np.random.PCG64(91 + page_size))
    B, Hq, Hkv, D = 6, 8, 2, 128
    L = np.array([700, 0, 129, 64, 2048, 33], np.int32)
    T = np.array([60, 7, 33, 1, 48, 72])
    w = wl.random_workload(1200 + page_size, B, Hq, Hkv, D, L, T, max_depth=10)
    k, v, cu, table = _in_cache_layout(w, rng, page_size)
    draft, target = make_tokens(rng, w.parent, w.cu_T, vocab=25, plant=0.9)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    i16 = lambda a: a.view(np.int16)
    q, cu_T, L_d, parent = dev(i16(w.q)), dev(w.cu_T), dev(L), dev(w.parent)
    k0, v0 = dev(i16(k)), dev(i16(v))
    k_d, v_d = k0.clone(), v0.clone()
    cu_d, table_d = dev(cu), dev(table)
    draft_d, target_d = dev(draft), dev(target)
    max_path = 12
    out = torch.empty(q.shape, dtype=torch.float32, device="cuda")
    lse = torch.empty(q.shape[:2], dtype=torch.float32, device="cuda")
    path = torch.full((B, max_path), -1, dtype=torch.int32, device="cuda")
    plen = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
    err = torch.zeros(1, dtype=torch.int32, device="cuda")
    args = binding.make_args(q=q, k_tree=None, v_tree=None, k_cache=k_d, v_cache=v_d, anc_mask=None, cu_T=cu_T, L=L_d,
                             max_T=w.max_T, max_L=w.max_L, scale=w.scale, cu_L=cu_d, page_table=table_d,
                             page_size=page_size, num_splits=3, out=out, lse=lse, parent=parent)
    ws = torch.empty((binding.workspace_bytes(args) + 3) // 4, dtype=torch.float32, device="cuda")
    args.workspace, args.workspace_bytes = ws.data_ptr(), ws.numel() * 4
    cargs = verify.make_commit_args(cu_T=cu_T, L=L_d, path=path, path_len=plen, k_tree=None, v_tree=None, k_cache=k_d,
                                    v_cache=v_d, cu_L=cu_d, page_table=table_d, page_size=page_size, L_out=L_out,
                                    err_flag=err)

    def one_pass(stream=None):
        binding.tree_verify_attn_raw(args, stream)
        verify.accept_greedy(parent, cu_T, draft_d, target_d, max_path, path=path, path_len=plen, next_token=nxt,
                             stream=stream)
        verify.commit_path_raw(cargs, stream)

    say(f"[case] whole pass eager, page_size={page_size}")
    one_pass()
    torch.cuda.synchronize()
    assert int(err.item()) == 0
    outputs = (out, lse, path, plen, nxt, L_out, k_d, v_d)
    eager = [t.clone() for t in outputs]
    paths, nxt_ref = vo.accept_greedy(w.parent, w.cu_T, draft, target, max_path=max_path)
    assert [list(path[b, :plen[b]].cpu().numpy()) for b in range(B)] == paths and nxt.cpu().tolist() == nxt_ref

    def reset():
        k_d.copy_(k0), v_d.copy_(v0)
        for t in (out, lse, plen, nxt, L_out):
            t.zero_()
        path.fill_(-1)

    reset()
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        one_pass(side)
    for replay in range(3):
        say(f"[case] whole pass, graph replay {replay}")
        reset()                                  # eager work between the replays
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert int(err.item()) == 0
        for name, got, want in zip("out lse path path_len next L_out k v".split(), outputs, eager):
            assert torch.equal(got, want), (name, replay)


@pytest.mark.parametrize("page_size", [0, 16])
def test_commit_of_an_8bit_cache(torch_dev, page_size):
    """One byte per element (the attention's kv_fp8 layout): copy commit and in-place commit move the same rows."""
    torch = torch_dev
    from paper_2510_26577_amd import verify
    rng = np.random.Generator(np.random.PCG64(95 + page_size))
    B, Hkv, D = 4, 2, 128
    T = np.array([30, 1, 9, 64])
    L = np.array([100, 0, 31, 5], np.int32)
    w = wl.random_workload(1500 + page_size, B, 4, Hkv, D, L, T, max_depth=9)
    w8, _, _ = wl.to_fp8_kv(w)
    k, v, cu, table = _in_cache_layout(w8, rng, page_size)
    k, v = k.astype(np.uint8), v.astype(np.uint8)
    paths = [sorted(rng.choice(int(t), size=int(min(t, 5)), replace=False).tolist()) for t in T]
    max_path = 8
    path = np.full((B, max_path), -1, np.int32)
    for b, pth in enumerate(paths):
        path[b, :len(pth)] = pth
    plen = np.array([len(pth) for pth in paths], np.int32)
    dev = lambda a: None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()
    at = lambda arr, b, t: arr[cu[b] + t] if page_size == 0 else arr[table[b, t // page_size], t % page_size]

    def expected(src_k, src_v, tree_k=None, tree_v=None):
        ek, ev = src_k.copy(), src_v.copy()
        for b, pth in enumerate(paths):
            for j, node in enumerate(pth):
                rk = at(src_k, b, L[b] + node) if tree_k is None else tree_k[w8.cu_T[b] + node]
                rv = at(src_v, b, L[b] + node) if tree_v is None else tree_v[w8.cu_T[b] + node]
                if page_size == 0:
                    ek[cu[b] + L[b] + j], ev[cu[b] + L[b] + j] = rk, rv
                else:
                    t = L[b] + j
                    ek[table[b, t // page_size], t % page_size], ev[table[b, t // page_size], t % page_size] = rk, rv
        return ek, ev

    for in_place in (True, False):
        say(f"[case] 8-bit commit page_size={page_size} in_place={in_place}")
        k_d, v_d = dev(k), dev(v)
        err = torch.zeros(1, dtype=torch.int32, device="cuda")
        L_out = torch.zeros(B, dtype=torch.int32, device="cuda")
        verify.commit_path(cu_T=dev(w8.cu_T), L=dev(L), path=dev(path), path_len=dev(plen),
                           k_tree=None if in_place else dev(w8.k_tree), v_tree=None if in_place else dev(w8.v_tree),
                           k_cache=k_d, v_cache=v_d, cu_L=dev(cu), page_table=dev(table), page_size=page_size,
                           L_out=L_out, err_flag=err)
        torch.cuda.synchronize()
        ek, ev = expected(k, v) if in_place else expected(k, v, w8.k_tree, w8.v_tree)
        assert int(err.item()) == 0
        assert np.array_equal(k_d.cpu().numpy(), ek) and np.array_equal(v_d.cpu().numpy(), ev)
        assert np.array_equal(L_out.cpu().numpy(), L + plen)


# ---- acceptance by speculative sampling ----

def run_sampling(torch, parent, cu_T, tok, p, q, u, uf, max_path, with_flag=True, misalign=False, workgroups=0, sum_T=0,
                 unit_rows=False):
    """workgroups: 0 = the library spreads a sequence over as many workgroups as it sees fit, 1 = one per sequence
    (no workspace passed, unless sum_T asks for the row sums ahead of the walk), 2 .. 16 = that many.
    sum_T: the host's count of nodes (0 = not given: no row sums ahead of the walk)."""
    from paper_2510_26577_amd import verify
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    flag = torch.zeros(1, dtype=torch.int32, device="cuda") if with_flag else None
    dp, dq = d(p, np.float32), d(q, np.float32)
    if misalign:                                 # the same rows, starting 4 bytes past a 16-byte boundary
        shifted = []
        for x in (dp, dq):
            flat = torch.empty(x.numel() + 1, dtype=torch.float32, device="cuda")
            flat[1:].copy_(x.reshape(-1))
            shifted.append(flat[1:].view(x.shape))
            assert shifted[-1].data_ptr() % 16 == 4
        dp, dq = shifted
    path, n, nxt = verify.accept_sampling(d(parent, np.int32), d(cu_T, np.int32), d(tok, np.int32), dp,
                                          dq, d(u, np.float32), d(uf, np.float32), max_path, err_flag=flag,
                                          workspace=None if workgroups == 1 and not sum_T else "auto",
                                          workgroups_per_sequence=workgroups, sum_T=sum_T, unit_rows=unit_rows)
    torch.cuda.synchronize()
    return path.cpu().numpy(), n.cpu().numpy(), nxt.cpu().numpy(), (int(flag.item()) if with_flag else 0)


def sampling_margin(parent, cu_T, tok, p, q, u, uf, paths, nxt, unit_rows=False):
    """Smallest relative distance of any decision the oracle took from its threshold (both sides decide in fp64 on the
    same fp32 data, but sum in different orders: a decision closer than that rounding to its threshold may differ)."""
    # the cases below are seeded: the margin is asserted, so a case on a threshold would be seen, not hidden
    worst = np.inf
    for b, path in enumerate(paths):
        t0, T = int(cu_T[b]), int(cu_T[b + 1] - cu_T[b])
        if T == 0:
            continue
        for cur in path:
            r = p[t0 + cur].astype(np.float64)
            Z = 1.0 if unit_rows else r.sum()
            qq = q[t0 + cur].astype(np.float64)
            for c in range(cur + 1, T):
                if parent[t0 + c] != cur:
                    continue
                x = int(tok[t0 + c])
                if r[x] > 0:
                    worst = min(worst, abs(float(u[t0 + c]) * qq[x] * Z - r[x]) / r[x])
                if c in path:
                    break
                r = np.maximum(0.0, r - Z * qq).astype(np.float32).astype(np.float64)
                Z = r.sum()
    return worst


@pytest.mark.parametrize("B,T_hi,V,temp,drift", [(1, 8, 1000, 1.0, 0.5), (4, 60, 32000, 1.0, 1.0), (33, 40, 4099, 0.7, 0.3),
                                                 (3, 25, 128256, 0.5, 0.2), (64, 12, 517, 1.5, 2.0), (5, 1, 64, 1.0, 1.0),
                                                 (2, 6, 7, 1.0, 1.0), (2, 1100, 64, 1.0, 0.3)])
def test_accept_sampling_matches_oracle(torch_dev, B, T_hi, V, temp, drift):
    """Paths, lengths and the drawn token equal the oracle's exactly on softmax-shaped distributions at vocabulary
    sizes from 7 to Llama 3's 128256 (several segments per wave and a ragged tail), ragged trees with empty ones
    and one longer than the kernel keeps in LDS, and path limits that cut the walk."""
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(1000 + B + T_hi + V))
    T = rng.integers(0 if B > 4 else 1, T_hi + 1, B)
    T[0] = T_hi
    cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    parent = np.concatenate([wl.tree_expand_prune(rng, int(t)) if t > 4 else wl.tree_uniform(rng, int(t), 4) if t > 0
                             else np.zeros(0, np.int32) for t in T]).astype(np.int32)
    p, q, tok, u, uf = wl.sampling_inputs(rng, parent, cu_T, V, temperature=temp, drift=drift)
    say(f"[case] accept_sampling B={B} T<={T_hi} V={V} temp={temp} drift={drift}")
    longest = 0
    for max_path, unit in ((int(T.max()) + 1, False), (3, False), (1, False), (int(T.max()) + 1, True), (2, True)):
        # unit: the target rows taken as distributions (a freshly reached node's normaliser is 1)
        ref_paths, ref_next = vo.accept_sampling(parent, cu_T, tok, p, q, u, uf, max_path=max_path, unit_rows=unit)
        assert sampling_margin(parent, cu_T, tok, p, q, u, uf, ref_paths, ref_next, unit_rows=unit) > 1e-9
        for workgroups in (0, 1, 2, 16) if max_path not in (2, 3) else (0, 1):
            if B * workgroups > 256:
                continue
            # the row sums made ahead of the walk (the host's node count given): the right count, one that is too
            # small (the trees past it are walked without) and one that is too large (no row is read past the last)
            for sum_T in (0, int(cu_T[-1])) + ((int(cu_T[-1]) // 2 + 1, int(cu_T[-1]) + 37) if workgroups in (0, 2) else ()):
                path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok, p, q, u, uf, max_path, workgroups=workgroups,
                                                  sum_T=sum_T, unit_rows=unit)
                case = (workgroups, sum_T, unit)
                assert flag == 0, case
                assert list(n) == [len(x) for x in ref_paths], case
                assert list(nxt) == ref_next, case
                for b, x in enumerate(ref_paths):
                    assert list(path[b, :len(x)]) == x, case
        longest = max(longest, max(len(x) for x in ref_paths))
        if max_path == 3 and not unit and V % 4 == 0:   # rows that do not start on 16 bytes take the one-element path
            path2, n2, nxt2, flag2 = run_sampling(torch, parent, cu_T, tok, p, q, u, uf, max_path, misalign=True)
            assert flag2 == 0 and np.array_equal(n, n2) and np.array_equal(nxt, nxt2) and np.array_equal(path, path2)
    if T_hi >= 8 and drift <= 1.0:
        assert longest >= 3                      # (the cases do accept drafted tokens)


def test_accept_sampling_rejections_reach_the_residual(torch_dev):
    """A star of children that the target gives no weight: every one is rejected, each rejection rewrites the residual,
    and the last token comes from the residual after all of them; with q = p every child is accepted at once."""
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(77))
    V, k, B = 3001, 9, 6
    parent = np.tile(np.array([-1] + [0] * k, np.int32), B)
    cu_T = (np.arange(B + 1) * (k + 1)).astype(np.int32)
    p, q, tok, u, uf = wl.sampling_inputs(rng, parent, cu_T, V, drift=1.5)
    for b in range(B):
        t0 = b * (k + 1)
        if b % 2 == 0:                           # no weight on the drafted tokens: all rejected
            p[t0, tok[t0 + 1:t0 + k + 1]] = 0.0
        else:                                    # q = p: the first child is accepted whatever u says
            q[t0] = p[t0]
            u[t0 + 1] = np.float32(0.999)
    ref_paths, ref_next = vo.accept_sampling(parent, cu_T, tok, p, q, u, uf)
    assert [len(x) for x in ref_paths] == [1, 2] * (B // 2)
    say(f"[case] accept_sampling star B={B} k={k} V={V}")
    for workgroups, sum_T in ((1, 0), (4, 0), (1, B * (k + 1)), (4, B * (k + 1))):
        path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok, p, q, u, uf, k + 1, workgroups=workgroups, sum_T=sum_T)
        assert flag == 0 and list(n) == [1, 2] * (B // 2) and list(nxt) == ref_next, (workgroups, sum_T)
    path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok, p, q, u, uf, k + 1)
    assert flag == 0 and list(n) == [1, 2] * (B // 2) and list(nxt) == ref_next
    for b in range(0, B, 2):
        assert nxt[b] not in set(tok[b * (k + 1) + 1:(b + 1) * (k + 1)])
    # without an error flag the call works the same
    path2, n2, nxt2, _ = run_sampling(torch, parent, cu_T, tok, p, q, u, uf, k + 1, with_flag=False)
    assert np.array_equal(n, n2) and np.array_equal(nxt, nxt2) and np.array_equal(path, path2)


def test_accept_sampling_flags_bad_input_and_leaves_other_sequences_alone(torch_dev):
    """A drafted token outside the vocabulary is never accepted and sets the flag to 1 + its sequence; a residual that
    vanishes (the draft distribution covers the target's whole weight and the drafted token is refused) sets it too and
    ends that sequence with token -1; the other sequences' results are the oracle's."""
    torch = torch_dev
    rng = np.random.Generator(np.random.PCG64(78))
    V = 50
    parent = np.array([-1, 0, 0, -1, 0, 1, -1, 0], np.int32)
    cu_T = np.array([0, 3, 6, 8], np.int32)
    p, q, tok, u, uf = wl.sampling_inputs(rng, parent, cu_T, V)
    ref_paths, ref_next = vo.accept_sampling(parent, cu_T, tok, p, q, u, uf)
    # sequence 1: its first child's token is not a token
    tok1 = tok.copy()
    tok1[4] = V + 5
    for workgroups, sum_T in ((1, 0), (2, 0), (1, 8), (2, 8)):
        path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok1, p, q, u, uf, 4, workgroups=workgroups, sum_T=sum_T)
        assert flag == 2 and n[1] == 1 and 0 <= nxt[1] < V, (workgroups, sum_T)
    path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok1, p, q, u, uf, 4)
    assert flag == 2
    assert [int(nxt[0]), int(nxt[2])] == [ref_next[0], ref_next[2]] and [int(n[0]), int(n[2])] == [len(ref_paths[0]), len(ref_paths[2])]
    assert n[1] == 1 and 0 <= nxt[1] < V         # nothing accepted below the root, the token drawn from the root's row
    # sequence 2: q = 2 p at the root (no distribution) and u = 1.5 refuse the child, and the residual max(0, p - q) is empty
    q2, u2 = q.copy(), u.copy()
    q2[6] = 2.0 * p[6]
    u2[7] = np.float32(1.5)
    with pytest.raises(ValueError):
        vo.accept_sampling(parent, cu_T, tok, p, q2, u2, uf)
    for workgroups, sum_T in ((1, 0), (2, 0), (1, 8), (2, 8)):
        path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok, p, q2, u2, uf, 4, workgroups=workgroups, sum_T=sum_T)
        assert flag == 3 and nxt[2] == -1 and n[2] == 1, (workgroups, sum_T)
    path, n, nxt, flag = run_sampling(torch, parent, cu_T, tok, p, q2, u2, uf, 4)
    assert flag == 3 and nxt[2] == -1 and n[2] == 1
    assert [int(nxt[0]), int(nxt[1])] == ref_next[:2]


def test_accept_sampling_waits_are_bounded(torch_dev):
    """The waits between the workgroups that share a sequence give up after a bounded number of polls: forced from the
    host (every wait expects one arrival more than there are workgroups, 64 polls), every workgroup leaves at its first
    wait, the kernel ends normally with the flag set, and the same inputs then run through as usual."""
    torch = torch_dev
    from paper_2510_26577_amd import verify
    rng = np.random.Generator(np.random.PCG64(79))
    B, V = 3, 20000
    T = np.array([9, 5, 7])
    cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    parent = np.concatenate([wl.tree_uniform(rng, int(t), 4) for t in T]).astype(np.int32)
    p, q, tok, u, uf = wl.sampling_inputs(rng, parent, cu_T, V)
    d = lambda a, t: torch.from_numpy(np.ascontiguousarray(a, dtype=t)).cuda()
    args = (d(parent, np.int32), d(cu_T, np.int32), d(tok, np.int32), d(p, np.float32), d(q, np.float32), d(u, np.float32),
            d(uf, np.float32), 6)
    say("[case] accept_sampling, waits that cannot complete (bounded at 64 polls)")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    verify.accept_sampling(*args, err_flag=flag, workgroups_per_sequence=4, wait_bound_test_spins=64)
    torch.cuda.synchronize()
    assert 1 <= int(flag.item()) <= B
    flag.zero_()
    path, n, nxt = verify.accept_sampling(*args, err_flag=flag, workgroups_per_sequence=4)
    torch.cuda.synchronize()
    ref_paths, ref_next = vo.accept_sampling(parent, cu_T, tok, p, q, u, uf, max_path=6)
    assert int(flag.item()) == 0 and list(nxt.cpu().numpy()) == ref_next
    assert list(n.cpu().numpy()) == [len(x) for x in ref_paths]
