"""C-ABI checks that need no GPU: the library loads, exports every symbol the
header declares, mirrors the argument struct, and its host-side validation and
split planning behave (those paths return before any launch)."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2510_26577_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        binding.build_library()
    return binding.load_library()


def declared_symbols(header="tva.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tva_[a-z_]+)\s*\(", text)))


def test_exports_match_header(lib):
    syms = declared_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None


def test_verify_exports_match_header(lib):
    from paper_2510_26577_amd import verify
    syms = declared_symbols("tva_verify.h")
    assert set(syms) == set(binding.VERIFY_EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None
    assert lib.tva_sizeof_commit_args() == ctypes.sizeof(verify.CommitArgs)


def test_draft_exports_match_header(lib):
    from paper_2510_26577_amd import draft
    syms = declared_symbols("tva_draft.h")
    assert set(syms) == set(binding.DRAFT_EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None
    draft._lib()
    assert lib.tva_sizeof_expand_args() == ctypes.sizeof(draft.ExpandArgs)
    # shapes are refused from host values alone: nothing is launched
    assert draft.expand_workspace_bytes(2, 128256, 12, 24) == 24 * (16 + 1) * 12 * 8
    for kw in (dict(K=17), dict(K=0), dict(V=4, K=5), dict(V=8192 * 40, K=16)):
        a = draft.ExpandArgs()
        a.B, a.V, a.K, a.sum_N = 1, kw.get("V", 1000), kw.get("K", 4), 3
        assert lib.tva_expand_workspace_bytes(ctypes.byref(a)) == ctypes.c_size_t(-1).value
        assert lib.tva_expand_layer(ctypes.byref(a), None) < 0
    assert lib.tva_tree_select_subtree(None, None, None, None, 1, 4096, None, None, None, None) == -2
    # nothing to do is not an error, and touches no pointer
    a = draft.ExpandArgs()
    a.B, a.V, a.K, a.sum_N, a.max_N = 0, 1000, 4, 0, 0
    assert lib.tva_expand_layer(ctypes.byref(a), None) == 0
    a.B = 3
    assert lib.tva_expand_layer(ctypes.byref(a), None) == 0          # three sequences without rows
    a.sum_N, a.max_N = 70000, 4
    assert lib.tva_expand_layer(ctypes.byref(a), None) == -2         # more rows than a grid dimension holds
    a.sum_N, a.max_N = 300, 300
    assert lib.tva_expand_layer(ctypes.byref(a), None) == -2         # 1200 candidates in one sequence
    assert lib.tva_tree_select_subtree(None, None, None, None, 0, 0, None, None, None, None) == 0


def test_host_exports_match_header(lib):
    syms = declared_symbols("tva_cast.h")
    assert set(syms) == set(binding.CAST_EXPORTS)
    for s in syms:
        assert getattr(lib, s) is not None


def test_microbenchmark_library_exports_match_header():
    """libtva_ubench (measurement aid, include/tva_ubench.h) loads and exports what its header declares."""
    from paper_2510_26577_amd import ubench
    if not os.path.exists(ubench.LIB_PATH):
        ubench.build_library()
    ul = ubench.load_library()
    syms = declared_symbols("tva_ubench.h")
    assert set(syms) == set(ubench.EXPORTS)
    for s in syms:
        assert getattr(ul, s) is not None


def test_struct_mirror_and_version(lib):
    assert lib.tva_sizeof_args() == ctypes.sizeof(binding.TvaArgs)
    assert lib.tva_version() == binding.EXPECTED_VERSION
    assert lib.tva_strerror(0) == b"ok" and b"workspace" in lib.tva_strerror(-3)


def shape_args(**kw):
    a = binding.TvaArgs()
    a.B, a.Hq, a.Hkv, a.D = 1, 32, 8, 128
    a.sum_T, a.max_T, a.mask_words, a.max_L = 60, 60, 1, 2048
    a.scale = 0.088
    for k, v in kw.items():
        setattr(a, k, v)
    return a


def test_plan_and_workspace(lib):
    a = shape_args(num_splits=1)
    assert binding.plan_splits(a) == 1 and binding.workspace_bytes(a) == 0
    a = shape_args(num_splits=4)
    assert binding.plan_splits(a) == 4
    assert binding.workspace_bytes(a) == 4 * 60 * 32 * 129 * 4
    a = shape_args(num_splits=1000)  # capped by the tile size
    s = binding.plan_splits(a)
    assert 1 <= s <= 2048 // 64
    a = shape_args(num_splits=0)
    assert binding.plan_splits(a) >= 1
    a = shape_args(max_L=0)
    assert binding.plan_splits(a) == 1


@pytest.mark.parametrize("B,L,T,rows,splits", [
    (1, 2048, 60, 64, 7),      # the headline shape: 32 natural workgroups of 64 rows; 7 splits of 5 tiles (224 workgroups:
                               # the tree's tile rides on the short last split) beat 8 of 4, whose last one has 5 as well
    (4, 2048, 60, 64, 2),      # 128 natural: one per CU (256) with splits of 16 tiles; 512 with 8 measures the same, with twice the partial rows
    (4, 4096, 60, 64, 4),
    (3, 2048, 60, 64, 5),      # 96 natural: on to 480
    (5, 2048, 60, 64, 3),      # 160 natural: 480
    (12, 2048, 8, 32, 5),      # the same for the 32-row shape: 96 natural -> 480
    (8, 2048, 60, 128, 2),     # 128 workgroups of 128 rows, two splits of 16 tiles
    (16, 2048, 60, 128, 1),    # 256 of them
    (8, 1024, 40, 64, 1),      # 128 of 128 rows would need splits of 8 tiles: 192 of 64 rows instead
    (20, 2048, 60, 256, 1),    # more than 256 of 128 rows: 160 of 256 rows, not split into a second round
    (32, 2048, 60, 256, 1),
    (4, 8192, 60, 256, 8),     # few sequences, many keys
    (8, 4096, 32, 256, 4),     # exactly 128 rows
    (16, 2048, 16, 64, 2),     # 64 rows: never the large shapes; 128 natural -> 256 (measured: 4 splits 12 % slower)
    (64, 2048, 8, 32, 1),      # 32 rows
    (2, 300, 8, 32, 3),        # five tiles: splits of 2, 2, 1 + the tree's own against six in a row
    (8, 512, 24, 64, 1),       # 128 workgroups, eight tiles: two splits would save four, a merge pass costs more
    (8, 768, 24, 64, 2),       # ... twelve tiles: two splits save six
    (1, 512, 8, 32, 8),        # eight tiles, eight natural workgroups: one tile per split (64 workgroups)
    (4, 512, 1, 32, 3),        # ... 32 natural: splits of one tile would take 256, so 3, 3, 2 + the tree's own
    (32, 2048, 9, 64, 1),      # 256 natural workgroups of 64 rows: every CU has one already, a split only adds the merge
    (16, 2048, 20, 64, 1),     # ... the same with two row blocks at batch 16
    (16, 2048, 9, 64, 4),      # 128 natural: split
])
def test_launch_plan_bands(lib, B, L, T, rows, splits):
    """The launch planner is host arithmetic on the shapes: one case per band of its rules (Hq 32, Hkv 8)."""
    a = shape_args(B=B, max_L=L, max_T=T, sum_T=B * T)
    assert (binding.plan_workgroup_rows(a), binding.plan_splits(a)) == (rows, splits)
    ck = binding.plan_chunk_keys(a)
    assert ck % 32 == 0 and ck * splits >= L > ck * (splits - 1)


def test_launch_plan_properties_over_the_cost_table_grid(lib):
    """The grid the attention cost tables are measured on (paper, Method: f(B, c, n) for c = k L, n = 1..N;
    here B = 1, 2, 4 and 8, c = 256..2048, n = 1..72, benchmark head shape).  Whatever the split count the
    planner settles on, a split keeps two tiles or more (one tile in launches of at most 128 workgroups over six
    tiles or more), splits of
    the small shapes stay within two workgroups per CU, the longest split (the tree's own tiles ride on the last one) is no longer than an unsplit pass
    would be minus what a merge pass costs, and the rows per workgroup never shrink as the tree grows."""
    for B in (1, 2, 4, 8):
        for c in range(256, 2049, 256):
            prev_rows = 0
            for n in range(1, 73):
                a = shape_args(B=B, max_L=c, max_T=n, sum_T=B * n, mask_words=(n + 63) // 64)
                rows, S, ck = binding.plan_workgroup_rows(a), binding.plan_splits(a), binding.plan_chunk_keys(a)
                assert rows >= prev_rows, (B, c, n, rows)
                prev_rows = rows
                if S == 1:
                    continue
                tiles, tree_tiles = -(-c // 64), -(-n // 64)
                wgs = B * 8 * -(-4 * n // rows) * S
                assert (ck >= 128 or (ck == 64 and wgs <= 128 and tiles >= 6)) and S == -(-c // ck), (B, c, n, S, ck)
                if rows <= 64:
                    assert wgs <= 512, (B, c, n, S)
                longest = max(ck // 64, tiles - (S - 1) * (ck // 64) + tree_tiles)
                assert tiles + tree_tiles - longest >= 3, (B, c, n, S, ck)


@pytest.mark.parametrize("kw,code", [
    (dict(D=96), -2), (dict(max_T=129, mask_words=3), -2), (dict(mask_words=0), -2),
    (dict(Hq=30), -1), (dict(B=0), -1), (dict(max_L=-1), -1), (dict(max_T=100, mask_words=1), -2),
    (dict(plan_shape=6), -1), (dict(plan_shape=-1), -1), (dict(sum_L=-5), -1),
    # query subsets: the plan and the workspace size are computed from sum_Q / max_Q, so they are checked
    # wherever those are (cu_Q is only tested for being set here, never read)
    (dict(cu_Q=8, sum_Q=-1, max_Q=4), -1), (dict(cu_Q=8, sum_Q=61, max_Q=4), -1), (dict(cu_Q=8, sum_Q=10, max_Q=61), -1),
])
def test_invalid_shapes_rejected_before_launch(lib, kw, code):
    a = shape_args(**kw)
    assert lib.tva_plan_splits(ctypes.byref(a)) == -1
    assert lib.tva_workspace_bytes(ctypes.byref(a)) == ctypes.c_size_t(-1).value
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == code
    assert lib.tva_tree_verify_attn_static(ctypes.byref(a), None) == code


def test_named_shapes_and_static_scratch_limit(lib):
    """plan_shape names the workgroup shape (rows per workgroup follow); the entry point that uses the
    library's own scratch array refuses, from the shapes alone, plans that need more than it holds."""
    for shape, rows in ((1, 32), (2, 64), (3, 64), (4, 128), (5, 256)):
        assert binding.plan_workgroup_rows(shape_args(plan_shape=shape)) == rows
    assert lib.tva_static_scratch_bytes() == binding.STATIC_SCRATCH_BYTES == 32 << 20
    big = shape_args(B=8, Hq=64, Hkv=8, max_T=128, mask_words=2, sum_T=8 * 128, max_L=4096, num_splits=4)
    assert binding.workspace_bytes(big) > binding.STATIC_SCRATCH_BYTES
    assert lib.tva_tree_verify_attn_static(ctypes.byref(big), None) == -3   # nothing queued, no pointer read


def test_launch_plan_invariants_over_random_shapes(lib):
    """Whatever the shapes: the splits cover max_L, are whole tiles of at least two tiles unless the cache is
    shorter, the workspace matches the split count, the workgroup size is one of the four, the length hint never
    lengthens a split, and a forced split count is honoured up to the tile limit."""
    rng = np.random.Generator(np.random.PCG64(20251026))
    for _ in range(3000):
        Hkv = int(rng.choice([1, 2, 4, 8, 16]))
        G = int(rng.choice([1, 2, 4, 7, 8, 16]))
        B = int(rng.choice([1, 2, 3, 5, 8, 13, 32, 64, 200]))
        T = int(rng.integers(1, 129))
        L = int(rng.choice([0, 1, 63, 64, 65, 500, 2048, 4097, 20000, 100000]))
        kw = dict(B=B, Hq=Hkv * G, Hkv=Hkv, D=int(rng.choice([64, 128])), max_T=T, sum_T=B * T,
                  mask_words=(T + 63) // 64, max_L=L)
        fp8 = bool(rng.integers(0, 2)) and kw["D"] == 128
        a = shape_args(kv_fp8=int(fp8), **kw)
        S, ck, rows = binding.plan_splits(a), binding.plan_chunk_keys(a), binding.plan_workgroup_rows(a)
        assert rows in (32, 64, 128, 256) and S >= 1 and ck % 32 == 0 and ck >= 32
        assert S * ck >= L and (S - 1) * ck < max(L, 1)
        if S > 1:
            assert ck >= 64            # no split shorter than two 32-key blocks
        n_rows = B * T * kw["Hq"]
        assert binding.workspace_bytes(a) == (0 if S == 1 else S * n_rows * (kw["D"] + 1) * 4)
        hinted = shape_args(kv_fp8=int(fp8), sum_L=max(1, (B * L) // 2), **kw)
        assert binding.plan_chunk_keys(hinted) <= ck
        forced = shape_args(kv_fp8=int(fp8), num_splits=3, **kw)
        assert binding.plan_splits(forced) == min(3, max(1, -(-L // binding.plan_chunk_keys(forced)))) or L == 0


def test_length_hint_shortens_long_splits_of_ragged_batches(lib):
    """Four sequences of up to 32768 cached tokens, 96000 in all: 8 splits of 4096 keys would leave a quarter of
    the workgroups without keys; with the sum known the splits shrink so that the non-empty ones still fit one
    round (ceil(L_b / c) summed over the batch <= 8 * 4 per KV head)."""
    a = shape_args(B=4, max_L=32768, max_T=48, sum_T=4 * 48)
    assert (binding.plan_splits(a), binding.plan_chunk_keys(a)) == (8, 4096)
    a = shape_args(B=4, max_L=32768, max_T=48, sum_T=4 * 48, sum_L=96000)
    c = binding.plan_chunk_keys(a)
    assert c == 3456 and binding.plan_splits(a) == 10 and c % 64 == 0
    assert 96000 / c + 4 <= 8 * 4                        # the bound the planner relies on
    assert binding.workspace_bytes(a) == 10 * 4 * 48 * 32 * 129 * 4
    # equal lengths (sum = B * max_L), short splits, one sequence, forced splits: the hint changes nothing
    for kw in (dict(B=4, max_L=32768, sum_L=4 * 32768), dict(B=4, max_L=2048, sum_L=5000),
               dict(B=1, max_L=32768, sum_L=20000), dict(B=4, max_L=32768, sum_L=96000, num_splits=8)):
        b = shape_args(max_T=48, sum_T=kw["B"] * 48, **kw)
        kw.pop("sum_L")
        assert binding.plan_chunk_keys(b) == binding.plan_chunk_keys(shape_args(max_T=48, sum_T=kw["B"] * 48, **kw))
    assert lib.tva_plan_splits(ctypes.byref(shape_args(sum_L=-1))) == -1     # the plan reads it: refused
    

def test_host_lengths_give_the_shortest_split_that_fits_one_round(lib):
    """With the lengths themselves (tva_args.L_host) the planner counts the non-empty splits instead of bounding
    them: the split length is the smallest multiple of 64 (at least 1024) with sum ceil(L_b / c) <= S * B, never
    longer than what the sum alone gives; nonsense lengths still give a valid plan."""
    import numpy as np
    L = np.array([18040, 28252, 25008, 32165], dtype=np.int32)
    kw = dict(B=4, max_L=int(L.max()), max_T=48, sum_T=4 * 48)
    by_sum = binding.plan_chunk_keys(shape_args(sum_L=int(L.sum()), **kw))
    a = shape_args(sum_L=int(L.sum()), **kw)
    a.L_host = L.ctypes.data_as(ctypes.c_void_p)
    c = binding.plan_chunk_keys(a)
    count = lambda c: int(np.sum(-(-L // c)))
    assert c % 64 == 0 and 1024 <= c <= by_sum and count(c) <= 32 and count(c - 64) > 32
    assert (by_sum, c) == (3712, 3584)
    assert binding.plan_splits(a) == -(-int(L.max()) // c)
    assert binding.workspace_bytes(a) == binding.plan_splits(a) * 4 * 48 * 32 * 129 * 4
    # without the sum the count alone does the same; equal lengths, one sequence and forced splits are unchanged
    b = shape_args(**kw)
    b.L_host = L.ctypes.data_as(ctypes.c_void_p)
    assert binding.plan_chunk_keys(b) == c
    for L2, extra in ((np.full(4, 32165, np.int32), {}), (L, dict(num_splits=8)), (L[3:], dict(B=1, sum_T=48))):
        d = shape_args(**{**kw, **extra})
        plain = binding.plan_chunk_keys(d)
        L2 = np.ascontiguousarray(L2)
        d.L_host = L2.ctypes.data_as(ctypes.c_void_p)
        assert binding.plan_chunk_keys(d) == plain
    for junk in (np.zeros(4, np.int32), np.full(4, -7, np.int32), np.full(4, 2 ** 31 - 1, np.int32)):
        d = shape_args(**kw)
        d.L_host = junk.ctypes.data_as(ctypes.c_void_p)
        ck = binding.plan_chunk_keys(d)
        assert ck % 64 == 0 and ck >= 1024 and binding.plan_splits(d) == -(-int(L.max()) // ck)


def test_slot_table_is_a_permutation_that_pairs_long_with_short(lib):
    """tva_args.L_host in an unsplit launch of 33 .. 64 sequences, 8 KV heads, at most 64 rows per KV head: the slot
    table is a permutation of the sequences whatever the lengths are (ties, zeros, nonsense); slots j and j + 32
    (one CU) hold the sequences of ranks r and 63 - r by length, the CUs with one slot the longest ones; every
    other launch leaves the order alone."""
    import numpy as np
    rng = np.random.Generator(np.random.PCG64(5))
    for n in list(range(33, 65)) + [64, 64]:
        L = rng.integers(0, 3000, size=n).astype(np.int32)
        if n % 5 == 0:
            L[: n // 2] = 777                                  # ties
        if n == 64:
            L = rng.integers(-2 ** 31, 2 ** 31 - 1, size=n).astype(np.int32)
        a = shape_args(B=n, max_L=3000, max_T=8, sum_T=8 * n)
        assert binding.plan_slot_sequences(a) == []            # no lengths given
        a.L_host = L.ctypes.data_as(ctypes.c_void_p)
        if binding.plan_splits(a) != 1:
            continue
        seq = binding.plan_slot_sequences(a)
        assert sorted(seq) == list(range(n)), n
        order = sorted(range(n), key=lambda i: (-int(L[i]), i))   # longest first, the lower index among equals
        rank = {s_: r for r, s_ in enumerate(order)}
        shared = n - 32
        for j in range(shared):
            assert rank[seq[j]] + rank[seq[j + 32]] == 63, (n, j)
        assert sorted(rank[seq[j]] for j in range(shared, 32)) == list(range(64 - n)), n
    L = np.arange(80, dtype=np.int32)
    for kw in (dict(B=32), dict(B=64, Hkv=4), dict(B=64, max_T=40, sum_T=64 * 40), dict(B=64, num_splits=2), dict(B=65, sum_T=65 * 8)):
        a = shape_args(**{**dict(max_L=3000, max_T=8, sum_T=8 * 64), **kw})
        a.L_host = L.ctypes.data_as(ctypes.c_void_p)
        assert binding.plan_slot_sequences(a) == [], kw
    assert lib.tva_plan_slot_sequences(ctypes.byref(shape_args()), None) == -1


def test_draft_stage_queries_of_one_or_two_sequences_take_32_row_workgroups(lib):
    """Queries restricted to the newest nodes (cu_Q), at most 48 rows per KV head, one or two sequences: 32-row
    workgroups; from there on, and for the verification's own calls, the 64-row shape as before."""
    import numpy as np
    dummy = np.zeros(4, np.int32)                              # (plan queries read shapes only)
    def rows(B, max_Q, with_cu_Q=True):
        a = shape_args(B=B, max_L=1024, max_T=60, sum_T=60 * B)
        if with_cu_Q:
            a.cu_Q, a.sum_Q, a.max_Q = dummy.ctypes.data_as(ctypes.c_void_p), max_Q * B, max_Q
        return binding.plan_workgroup_rows(a)
    assert rows(1, 12) == 32 and rows(2, 12) == 32 and rows(1, 9) == 32
    assert rows(3, 12) == 64 and rows(8, 12) == 64 and rows(1, 13) == 64
    assert rows(1, 8) == 32                                    # (32 rows or fewer: as always)
    assert rows(1, 12, with_cu_Q=False) >= 64                  # all 60 nodes as queries: 240 rows


def test_fp8_arguments_checked_on_the_host(lib):
    assert binding.plan_splits(shape_args(kv_fp8=1)) >= 1                         # D = 128: fine
    a = shape_args(kv_fp8=1, D=64)
    assert lib.tva_plan_splits(ctypes.byref(a)) == -1 and lib.tva_tree_verify_attn(ctypes.byref(a), None) == -2
    a = shape_args(kv_fp8=2)
    assert lib.tva_plan_splits(ctypes.byref(a)) == -1 and lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1
    # the four shapes the 8-bit path has: 32, 64, 128 or 256 rows, like the 16-bit planner's bands
    for B, T, rows in [(1, 60, 64), (16, 60, 128), (32, 60, 256), (64, 8, 32)]:
        assert binding.plan_workgroup_rows(shape_args(kv_fp8=1, B=B, max_T=T, sum_T=B * T)) == rows


def test_null_pointers_and_cache_form_rejected(lib):
    a = shape_args()
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1      # null tensors
    a = shape_args(scale=0.0)
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1      # scale must be > 0
    for f in ("cu_T", "L", "q", "k_tree", "v_tree", "anc_mask", "out", "lse", "k_cache", "v_cache"):
        setattr(a, f, 0x1000)  # never dereferenced: the call fails validation first
    a.scale = 0.1
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1      # neither cache form
    a.cu_L = 0x1000
    a.page_table = 0x1000
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1      # both cache forms
    a.cu_L = None
    a.page_size, a.max_pages = 16, 4                                   # 64 tokens < max_L
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1
    a.max_pages = 128
    a.stride_tok = 1001                                                # not 16-byte aligned rows
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -1
    a.stride_tok = 0
    a.num_splits = 4                                                   # workspace missing
    assert lib.tva_tree_verify_attn(ctypes.byref(a), None) == -3


def test_mask_and_merge_argument_checks(lib):
    assert lib.tva_build_ancestor_mask(None, None, 1, 8, 1, None, None, None) == -1
    assert lib.tva_build_ancestor_mask(None, None, 0, 8, 1, None, None, None) == 0   # empty batch
    assert lib.tva_build_ancestor_mask(0x1000, 0x1000, 1, 100, 1, 0x1000, None, None) == -1
    assert lib.tva_merge_splits(None, None, 2, 4, 128, None, None, None) == -1
    assert lib.tva_merge_splits(0x1000, 0x1000, 2, 4, 96, 0x1000, 0x1000, None) == -2
    assert lib.tva_merge_splits(None, None, 2, 0, 128, None, None, None) == 0


def test_no_oracle_in_product_path():
    """The product package never imports the oracle, and vice versa."""
    pkg = os.path.join(ROOT, "paper_2510_26577_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                txt = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+\.*oracle", txt, flags=re.M), f
                assert "tva_oracle" not in txt and "libtva_oracle" not in txt, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            txt = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_26577_amd" not in txt and "libtva.so" not in txt and "tva.h" not in txt


def test_host_mask_builder_matches_oracle_and_validates(lib):
    """The host variant of the mask builder against the oracle's masks, and its synchronous tree check."""
    import numpy as np
    from oracle import tva_oracle as orc
    from paper_2510_26577_amd import workloads as wl
    rng = np.random.Generator(np.random.PCG64(5))
    T = [1, 9, 64, 65, 128, 0, 33]
    parent = np.concatenate([wl.tree_uniform(rng, t, 13) if t else np.zeros(0, np.int32) for t in T]).astype(np.int32)
    cu_T = np.concatenate([[0], np.cumsum(T)]).astype(np.int32)
    parent[cu_T[4] + 40] = -1                                   # a second root
    mask, rc, bad = binding.build_ancestor_mask_host(parent, cu_T, 128)
    assert rc == 0 and bad == -1
    assert np.array_equal(mask, orc.ancestor_mask(parent, cu_T, words=2))
    broken = parent.copy()
    broken[cu_T[2] + 7] = 7                                     # points at itself
    broken[cu_T[3] + 3] = 50                                    # points forward (a later node is also broken)
    _, rc, bad = binding.build_ancestor_mask_host(broken, cu_T, 128)
    assert rc == -5 and bad == cu_T[2] + 7
    assert lib.tva_strerror(-5).startswith(b"malformed tree")
    with pytest.raises(binding.TvaError):
        binding.build_ancestor_mask_host(parent, cu_T, 64)      # max_T below the largest tree
