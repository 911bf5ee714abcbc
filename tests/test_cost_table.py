"""The measured attention cost tables (profiles/attention_cost_table_B*.txt, written by
paper_2510_26577_amd.cost_table on an MI355X) drive the tree-size selection: file round trip,
conditioning for Algorithm 1, native selection against the oracle on the measured costs, and the
behaviour the method is built on -- costlier verification (bigger batch, longer context) keeps
fewer tree nodes.  A GPU case measures a tiny table."""
import os

import numpy as np
import pytest

from oracle import cast_oracle as co
from paper_2510_26577_amd import binding, cast, cost_table

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
L_GRID, M_ROWS = 256, 8


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(binding.LIB_PATH):
        binding.build_library()
    return binding.load_library()


def measured(B):
    return cost_table.read_table(os.path.join(ROOT, "profiles", f"attention_cost_table_B{B}.txt"))


def tree_scores(rng, n):
    parent = [-1] + [int(rng.integers(max(0, i - 6), i)) for i in range(1, n)]
    s = [1.0] * n
    for i in range(1, n):
        s[i] = s[parent[i]] * float(rng.uniform(0.1, 0.9))
    return np.array(s, np.float32)


def test_table_file_round_trip(tmp_path):
    t = np.arange(24, dtype=np.float64).reshape(3, 8) * 1.25 + 3
    path = str(tmp_path / "t.txt")
    cost_table.write_table(path, t, B=2, L=64, header_lines=["a header"])
    assert np.allclose(cost_table.read_table(path), t, atol=5e-4)
    assert open(path).readline().startswith("# a header")


def test_conditioning_makes_rows_strictly_increasing():
    t = np.array([[5.0, 4.0, 4.5, 7.0], [1.0, 1.0, 1.0, 0.5]])
    m = cost_table.make_strictly_increasing(t, eps=0.25, max_raise=10.0)
    assert np.all(np.diff(m, axis=1) > 0) and np.all(m >= t)
    assert np.allclose(m, [[5.0, 5.25, 5.5, 7.0], [1.0, 1.25, 1.5, 1.75]])
    with pytest.raises(ValueError, match="dips by"):             # a 25 % dip is no measurement noise
        cost_table.make_strictly_increasing(t, eps=0.25)
    small = np.array([[10.0, 9.8, 10.3]])                        # a 2 % one is
    assert np.allclose(cost_table.make_strictly_increasing(small), [[10.0, 10.001, 10.3]])
    inc = np.cumsum(np.ones((2, 5)), axis=1)
    assert np.array_equal(cost_table.make_strictly_increasing(inc), inc)     # already increasing: untouched


def test_measured_tables_are_plausible():
    for B in (1, 8):
        t = measured(B)
        assert t.shape == (M_ROWS, 72) and np.isfinite(t).all() and (t > 1.0).all() and (t < 1000.0).all()
        assert t[:, -1].mean() > t[:, 0].mean()                 # 72 tokens cost more than 1
    assert measured(8)[-1, -1] > measured(1)[-1, -1]            # so does a bigger batch


def test_selection_on_measured_costs_native_equals_oracle_and_shrinks_with_cost():
    rng = np.random.Generator(np.random.PCG64(3))
    tables = {B: cost_table.make_strictly_increasing(measured(B)) for B in (1, 8)}
    totals = {}
    for B in (1, 8):
        trees = np.stack([tree_scores(rng, 100) for _ in range(B)])
        counts = []
        for C3 in (0.5, 1.0, 2.0, 4.0, 8.0):
            for n0 in (100, 1000, 2000):
                k = cast.rerank_count(trees, tables[B], n0, L_GRID, 72, C3)
                assert k == co.rerank_count(trees, tables[B], n0, L_GRID, M_ROWS, 72, C3)
                assert 1 <= k <= 72
                counts.append(k)
        per_threshold = np.array(counts).reshape(5, 3).sum(axis=1)
        assert np.all(np.diff(per_threshold) <= 0)              # a higher threshold never keeps more
        totals[B] = int(np.sum(counts))
    assert totals[8] < totals[1]                                # batch 8 verifies fewer nodes than batch 1


@pytest.mark.gpu
def test_measure_tiny_table_on_gpu():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    t = cost_table.measure(B=2, L=128, M=2, N=16, copies=4, replays=3, n_values=[1, 8, 16])
    assert t.shape == (2, 16) and np.isfinite(t).all() and (t > 1.0).all() and (t < 500.0).all()
    m = cost_table.make_strictly_increasing(t, max_raise=1.0)   # (three replays of four copies: plumbing, not a measurement)
    k = cast.select_max_valid_index(np.cumsum(np.linspace(1.0, 0.1, 16)), m[0] / m[0, 0], 0.5)
    assert 1 <= k <= 16
