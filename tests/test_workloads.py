"""Seeded input generators: determinism, tree validity, shapes (CPU only)."""
import os

import numpy as np
import pytest

from oracle import tva_oracle as orc
from paper_2510_26577_amd import workloads as wl


def depth_of(par):
    d = np.zeros(len(par), dtype=np.int64)
    for i, p in enumerate(par):
        assert -1 <= p < i
        d[i] = 0 if p < 0 else d[p] + 1
    return d


def trees_of(w):
    return [w.parent[w.cu_T[b]:w.cu_T[b + 1]] for b in range(w.B)]


def test_config1_shape_and_tree():
    w = wl.config1()
    assert (w.B, w.Hq, w.Hkv, w.D, int(w.L[0]), int(w.T[0])) == (1, 4, 4, 64, 128, 8)
    par = trees_of(w)[0]
    assert par[0] == -1 and depth_of(par).max() <= 4
    assert all(max(0, i - 3) <= par[i] <= i - 1 for i in range(1, 8))
    assert w.scale == pytest.approx(1 / 8)


def test_config2_tree_is_parent_closed_prune():
    w = wl.config2()
    assert (w.Hq, w.Hkv, w.D, int(w.L[0]), int(w.T[0])) == (32, 8, 128, 2048, 60)
    par = trees_of(w)[0]
    d = depth_of(par)
    assert (par == -1).sum() == 1 and d.max() <= 6
    assert np.bincount(par[1:]).max() <= 4


@pytest.mark.parametrize("B", [1, 4, 16, 64])
def test_config3_sweep(B):
    w = wl.config3(B)
    assert w.B == B and np.all(w.T == wl.SWEEP[B])
    assert w.L.min() >= 512 and w.L.max() <= 2048
    assert max(depth_of(t).max() for t in trees_of(w)) <= 8
    assert w.k_cache.shape == (int(w.L.sum()), 8, 128)


def test_config4():
    w = wl.config4()
    assert (w.B, w.Hq, w.Hkv, w.G) == (8, 64, 8, 8) and np.all(w.L == 4096) and np.all(w.T == 32)
    assert max(depth_of(t).max() for t in trees_of(w)) <= 6


def test_config5_small_instance_page_table():
    w = wl.config5(l_lo=100, l_hi=200)  # same recipe, short lengths
    assert w.paged and w.page_size == 16 and w.B == 4
    used = []
    for b in range(4):
        n = (int(w.L[b]) + 15) // 16
        used += list(w.page_table[b, :n])
        assert np.all(w.page_table[b, n:] == -1)
    assert len(set(used)) == len(used) and max(used) < w.k_cache.shape[0]
    assert w.k_cache.shape[0] == int(np.ceil(1.25 * len(used)))
    assert max(depth_of(t).max() for t in trees_of(w)) <= 7


def test_determinism():
    a, b = wl.config3(4), wl.config3(4)
    for f in ("L", "parent", "q", "k_tree", "v_cache"):
        assert np.array_equal(getattr(a, f), getattr(b, f))


def test_values_look_standard_normal():
    w = wl.config2()
    x = wl.bf16_bits_to_f32(w.k_cache).astype(np.float64)
    assert abs(x.mean()) < 5e-3 and abs(x.std() - 1) < 5e-3


def test_golden_config1_fixture_matches_oracle():
    """Drift check of oracle + input recipe against the stored fixture (written by
    tests/golden/make_golden.py from the oracle alone)."""
    path = os.path.join(os.path.dirname(__file__), "golden", "cfg1_oracle.txt")
    w = wl.config1()
    out, lse = orc.tree_verify_attn(w)
    n = 0
    for line in open(path):
        if line.startswith("#"):
            continue
        f = line.split()
        i, h = int(f[0]), int(f[1])
        got = [lse[i, h], out[i, h, 0], out[i, h, 1], out[i, h, 62], out[i, h, 63]]
        np.testing.assert_allclose(got, [float(x) for x in f[2:]], rtol=1e-12, atol=1e-14)
        n += 1
    assert n == 32
