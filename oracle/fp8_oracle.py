"""CPU oracle of the attention with an 8-bit floating point KV cache.  TEST INFRASTRUCTURE ONLY:
imported by tests/ and nothing else; shares no code with the HIP path.

The paper does not quantise the cache; this variant is a widening of the kernel, and its definition
is the plain one: the stored bytes are OCP 8-bit floating point, format E4M3 (1 sign, 4 exponent,
3 mantissa bits, bias 7, no infinities, the all-ones magnitude 0x7F is NaN, magnitudes below 2^-6
are subnormal steps of 2^-9), K = k_scale * decode(k8), V = v_scale * decode(v8) with one scale per
tensor, and the attention is the paper's tree-masked softmax attention (Tree Reranking Phase: a node
attends to the committed tokens and to its own ancestors) on those K and V.

Every E4M3 value is k * 2^-9 with |k| <= 2^9 * 448, hence exactly a bf16 value: the oracle decodes
the bytes, re-expresses them as bf16 bit patterns (no rounding happens) and hands them to the bf16
attention oracle with scale * k_scale as the score scale; the output is multiplied by v_scale.
Pins: the paper has no such variant, so no expected value is taken from it; the decoder is pinned to the
format's published values and structure, the attention part is the pinned bf16 oracle.
"""
from __future__ import annotations

import dataclasses

import numpy as np

from . import tva_oracle


def e4m3_decode_table() -> np.ndarray:
    """float64[256]: value of every byte, written out from the format's definition."""
    out = np.empty(256, np.float64)
    for code in range(256):
        sign = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            out[code] = np.nan
        elif e == 0:
            out[code] = sign * (m / 8.0) * 2.0 ** -6
        else:
            out[code] = sign * (1.0 + m / 8.0) * 2.0 ** (e - 7)
    return out


def e4m3_decode(codes: np.ndarray) -> np.ndarray:
    return e4m3_decode_table()[np.asarray(codes, np.uint8)]


def _as_bf16_bits(x: np.ndarray) -> np.ndarray:
    """bf16 bit patterns of values that are exactly representable (checked)."""
    f = x.astype(np.float32)
    bits = f.view(np.uint32)
    if np.any(bits & 0xFFFF):
        raise ValueError("value is not a bf16 number")
    return (bits >> 16).astype(np.uint16)


def tree_verify_attn_fp8(w, k_scale: float, v_scale: float, rows=None):
    """w: a workload whose k_cache / v_cache / k_tree / v_tree hold uint8 E4M3 bytes (q stays bf16 bits).
    Returns (out float64 [sum_T, Hq, D], lse float64 [sum_T, Hq]) or the sampled rows' results."""
    dec = {}
    for name in ("k_cache", "v_cache", "k_tree", "v_tree"):
        v = e4m3_decode(getattr(w, name))
        if np.isnan(v).any():
            raise ValueError("NaN code in " + name)
        dec[name] = _as_bf16_bits(v)
    w16 = dataclasses.replace(w, scale=float(w.scale) * float(k_scale), **dec)
    out, lse = tva_oracle.tree_verify_attn(w16, rows=rows) if rows is not None else tva_oracle.tree_verify_attn(w16)
    return out * float(v_scale), lse
