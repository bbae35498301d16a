"""CPU oracle of the 8-bit prefix KV cache variant of the verification step.

TEST INFRASTRUCTURE ONLY (same rules as eagle2_oracle.py: imported by tests, the
smoke check and the benchmark's cpu-baseline leg; shares no code with the HIP path).

PARITY UNPINNED BY THE PAPER: the paper keeps its KV cache in the models' 16-bit
type (Appendix "Implementation Details" only says the cache is pre-allocated).  This
variant stores the *prefix* keys and values as 8-bit floating point with one float
scale per KV head; the tree's own keys and values stay 16-bit until they are
committed.  What is pinned is the number format (against the published table of the
format and against an independent library conversion) and, through eagle2_oracle's
tree_attn and commit_kv, the rest of the arithmetic.

Number format (OCP 8-bit floating point specification, E4M3): 1 sign bit, 4
exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds subnormals
(m/8 * 2^-6); there are no infinities; S.1111.111 is NaN; the largest finite value
is S.1111.110 = 448.
"""
from __future__ import annotations

import numpy as np

E4M3_MAX = 448.0


def e4m3_decode(codes) -> np.ndarray:
    """Value of every 8-bit code, float64 (NaN for 0x7f and 0xff)."""
    c = np.asarray(codes).astype(np.int64)
    sign = np.where((c >> 7) & 1, -1.0, 1.0)
    e = (c >> 3) & 15
    m = c & 7
    normal = np.ldexp(1.0 + m / 8.0, (e - 7).astype(np.int64))
    sub = np.ldexp(m / 8.0, -6)
    v = sign * np.where(e == 0, sub, normal)
    return np.where((e == 15) & (m == 7), np.nan, v)


def e4m3_encode(x) -> np.ndarray:
    """Nearest finite E4M3 value of every element, by exhaustive search: the value is
    first clamped to [-448, 448] (saturation), then the closest of the 127 finite
    magnitudes wins; a value exactly half-way between two neighbours goes to the one
    whose last mantissa bit is 0 (round to nearest even).  The sign is kept, also
    for zero.  Inputs must be finite."""
    x = np.asarray(x, dtype=np.float64)
    mags = e4m3_decode(np.arange(127))                  # codes 0x00 .. 0x7e: increasing magnitudes
    a = np.minimum(np.abs(x), E4M3_MAX)
    out = np.zeros(x.shape, dtype=np.uint8)
    flat_a, flat_o = a.reshape(-1), out.reshape(-1)
    for i, v in enumerate(flat_a):
        dist = np.abs(mags - v)
        best = np.flatnonzero(dist == dist.min())       # one code, or two neighbours on a tie
        code = int(best[0])
        if len(best) == 2 and (code & 1):
            code = int(best[1])
        flat_o[i] = code
    neg = np.signbit(x)
    return np.where(neg, out | 0x80, out).astype(np.uint8)


def dequantize(codes, scale) -> np.ndarray:
    """codes [T, Hkv, dh] with one scale per KV head -> float64 values code_value * scale[h]."""
    s = np.asarray(scale, dtype=np.float64)
    return e4m3_decode(codes) * s[None, :, None]


def quantize_rows(x, scale) -> np.ndarray:
    """x [..., Hkv, dh] -> codes of x / scale[h].  The quotient is taken in float32 (one
    correctly rounded division of the float32 images of x and of the scale), so that the
    rounding to 8 bits is decided on the same number on both sides of a comparison."""
    q = np.asarray(x, dtype=np.float32) / np.asarray(scale, dtype=np.float32)[:, None]
    return e4m3_encode(q.astype(np.float64))


def commit_kv_fp8(K_cache, V_cache, region_start: int, region_end: int, prefix_len: int,
                  K_tree, V_tree, path, k_scale, v_scale) -> int:
    """eagle2_oracle.commit_kv for an 8-bit cache: the accepted rows (root first) are
    quantised with the cache's per-head scales on their way in.  K_cache/V_cache are uint8
    code arrays [T, Hkv, dh]; returns the new prefix length."""
    n = int(prefix_len)
    for row in path:
        dst = region_start + n
        if dst >= region_end:
            break
        K_cache[dst] = quantize_rows(K_tree[int(row)], k_scale)
        V_cache[dst] = quantize_rows(V_tree[int(row)], v_scale)
        n += 1
    return n
