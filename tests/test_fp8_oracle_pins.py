"""Pins of the 8-bit floating point (OCP E4M3) decoder the fp8-KV oracle uses, against values the
format's specification fixes, and of the oracle itself against the bf16 oracle on inputs where the
two must agree exactly."""
import numpy as np
import pytest

from oracle import fp8_oracle as f8
from oracle import tva_oracle as orc
from paper_2510_26577_amd import workloads as wl


def test_decoder_against_the_values_the_format_fixes():
    t = f8.e4m3_decode_table()
    # OCP 8-bit floating point specification, E4M3: bias 7, subnormal step 2^-9, largest finite 448, no inf
    fixed = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 7 * 2.0 ** -9, 0x08: 2.0 ** -6, 0x0F: 1.875 * 2.0 ** -6,
             0x30: 0.5, 0x38: 1.0, 0x39: 1.125, 0x3C: 1.5, 0x40: 2.0, 0x44: 3.0, 0x48: 4.0, 0x77: 240.0,
             0x78: 256.0, 0x7E: 448.0, 0xB8: -1.0, 0xC0: -2.0, 0xFE: -448.0, 0x81: -2.0 ** -9}
    for code, value in fixed.items():
        assert t[code] == value, hex(code)
    assert t[0x80] == 0.0 and np.signbit(t[0x80])
    assert np.isnan(t[0x7F]) and np.isnan(t[0xFF]) and np.isnan(t).sum() == 2
    pos = t[:0x7F]
    assert np.all(np.diff(pos) > 0)                        # codes are ordered like their values
    assert np.array_equal(t[0x80:0xFF], -pos)              # sign bit only flips the sign
    assert np.array_equal(pos * 512, np.round(pos * 512))  # every value is a multiple of 2^-9
    # spacing doubles with every exponent step: 8 codes per binade
    assert np.allclose(pos[16:] / pos[8:-8], 2.0)


def test_quantiser_and_decoder_round_trip():
    """Two independently written tables: the input generator's encoder must invert the oracle's decoder."""
    t = f8.e4m3_decode_table()
    codes = np.array([c for c in range(256) if c not in (0x7F, 0xFF)], np.uint8)
    back = wl.f32_to_e4m3(t[codes].astype(np.float32))
    same = (back == codes) | ((codes == 0x80) & (back == 0x80))
    assert same.all()
    # nearest with ties to even, and saturation
    assert wl.f32_to_e4m3(np.array([1.0625, 1.1875, 1000.0, -1000.0, 2.0 ** -10], np.float32)).tolist() == \
        [0x38, 0x3A, 0x7E, 0xFE, 0x00]


def test_fp8_oracle_equals_bf16_oracle_on_values_both_can_hold():
    """K and V restricted to E4M3 values: the fp8 oracle on their codes, with scales that are powers of two,
    must equal the bf16 oracle on K * k_scale and V * v_scale (exact in bf16) with the plain scale."""
    w = wl.random_workload(4242, 3, 8, 2, 64, [70, 0, 33], [9, 5, 17], max_depth=5)
    rng = np.random.Generator(np.random.PCG64(7))
    codes = {}
    for name in ("k_cache", "v_cache", "k_tree", "v_tree"):
        c = rng.integers(0, 0x68, getattr(w, name).shape).astype(np.uint8)      # magnitudes up to 60
        codes[name] = c | (rng.integers(0, 2, c.shape).astype(np.uint8) << 7)
    import dataclasses
    w8 = dataclasses.replace(w, **codes)
    ks, vs = 0.25, 2.0
    o8, l8 = f8.tree_verify_attn_fp8(w8, ks, vs)
    as_bf16 = lambda name, sc: wl.f32_to_bf16_bits((f8.e4m3_decode(codes[name]) * sc).astype(np.float32))
    w16 = dataclasses.replace(w, k_cache=as_bf16("k_cache", ks), k_tree=as_bf16("k_tree", ks),
                              v_cache=as_bf16("v_cache", vs), v_tree=as_bf16("v_tree", vs))
    o16, l16 = orc.tree_verify_attn(w16)
    assert np.allclose(o8, o16, rtol=0, atol=1e-12) and np.allclose(l8, l16, rtol=0, atol=1e-12)


def test_nan_codes_are_refused():
    w = wl.random_workload(4243, 1, 4, 2, 64, [5], [3])
    w8, ks, vs = wl.to_fp8_kv(w)
    w8.k_cache.reshape(-1)[0] = 0x7F
    with pytest.raises(ValueError):
        f8.tree_verify_attn_fp8(w8, ks, vs)


def test_quantised_workload_stays_close_to_the_original():
    """Sanity of the input recipe: per-tensor scaling to 448 keeps the attention output within a few percent."""
    w = wl.random_workload(4244, 2, 8, 2, 128, [200, 64], [20, 8])
    w8, ks, vs = wl.to_fp8_kv(w)
    assert w8.k_cache.dtype == np.uint8 and w8.k_cache.shape == w.k_cache.shape
    o8, _ = f8.tree_verify_attn_fp8(w8, ks, vs)
    o16, _ = orc.tree_verify_attn(w)
    assert np.abs(o8 - o16).max() < 0.15 and np.abs(o8 - o16).mean() < 0.02
