"""Pins of the 8-bit KV oracle: the number format against the values its published
specification tabulates and against an independent library conversion (PyTorch's
float8_e4m3fn on the CPU); the commit step against the 16-bit one."""
import numpy as np
import pytest
import torch

from oracle import eagle2_oracle as orc
from oracle import fp8_kv_oracle as f8


def test_decode_matches_the_format_table():
    # OCP 8-bit floating point specification, E4M3 column of the value table
    table = {0x00: 0.0, 0x01: 2.0 ** -9, 0x07: 0.875 * 2.0 ** -6, 0x08: 2.0 ** -6, 0x38: 1.0, 0x39: 1.125,
             0x40: 2.0, 0x7e: 448.0, 0x78: 256.0, 0x81: -(2.0 ** -9), 0xb8: -1.0, 0xfe: -448.0}
    for code, val in table.items():
        assert f8.e4m3_decode(np.array([code]))[0] == val
    assert np.isnan(f8.e4m3_decode(np.array([0x7f, 0xff]))).all()
    assert np.signbit(f8.e4m3_decode(np.array([0x80]))[0])


def test_decode_matches_library_for_every_code():
    codes = np.arange(256, dtype=np.uint8)
    lib = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    mine = f8.e4m3_decode(codes)
    assert np.array_equal(np.isnan(lib), np.isnan(mine))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok], mine[ok])
    assert np.all(np.diff(mine[:127]) > 0)             # magnitudes increase with the code


def test_encode_is_identity_on_representable_values_and_monotone():
    codes = np.concatenate([np.arange(0, 127), np.arange(128, 255)]).astype(np.uint8)
    assert np.array_equal(f8.e4m3_encode(f8.e4m3_decode(codes)), codes)
    xs = np.linspace(-460.0, 460.0, 4001)
    vals = f8.e4m3_decode(f8.e4m3_encode(xs))
    assert np.all(np.diff(vals) >= 0)
    assert np.all(np.abs(vals - np.clip(xs, -448, 448)) <= np.maximum(np.abs(xs) * 2.0 ** -4, 2.0 ** -10))


def test_encode_ties_and_saturation():
    # half-way cases go to the even mantissa; beyond 448 saturates (the library returns NaN there)
    cases = [(1.0625, 0x38), (1.1875, 0x3a), (17.0, 0x58), (19.0, 0x5a), (432.0, 0x7e), (2.0 ** -10, 0x00),
             (1.5 * 2.0 ** -9, 0x02), (2.5 * 2.0 ** -9, 0x02), (464.0, 0x7e), (465.0, 0x7e), (1e6, 0x7e), (-1e6, 0xfe),
             (np.nextafter(np.float32(2.0 ** -10), np.float32(1.0)), 0x01), (0.0, 0x00), (-0.0, 0x80), (-1.1875, 0xba)]
    for x, code in cases:
        assert f8.e4m3_encode(np.array([x]))[0] == code, (x, code)


def test_encode_matches_library_in_range():
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(size=3000) * 3.0, rng.normal(size=1000) * 0.01, rng.uniform(-448, 448, 1000),
                        # every half-way point between neighbours, and its float32 neighbours
                        (f8.e4m3_decode(np.arange(126)) + f8.e4m3_decode(np.arange(1, 127))) / 2]).astype(np.float32)
    x = np.concatenate([x, np.nextafter(x, np.float32(np.inf)), np.nextafter(x, np.float32(-np.inf))])
    x = x[np.abs(x) <= 448]
    lib = torch.from_numpy(x.copy()).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    mine = f8.e4m3_encode(x.astype(np.float64))
    assert np.array_equal(lib, mine)


def test_quantize_rows_uses_the_heads_scale():
    rng = np.random.default_rng(4)
    x = rng.normal(size=(5, 3, 8)).astype(np.float32)
    scale = np.array([0.5, 1.0, 0.03125], dtype=np.float32)
    codes = f8.quantize_rows(x, scale)
    for h in range(3):
        assert np.array_equal(codes[:, h], f8.e4m3_encode(x[:, h].astype(np.float64) / float(scale[h])))   # power-of-two scales: exact quotients
    back = f8.dequantize(codes.reshape(5, 3, 8), scale)
    clipped = np.clip(x, -448 * scale[None, :, None], 448 * scale[None, :, None])
    assert np.all(np.abs(back - clipped) <= np.maximum(np.abs(clipped) * 2.0 ** -4, scale[None, :, None] * 2.0 ** -10))


def test_commit_kv_fp8_follows_the_16_bit_commit():
    """Same rows land in the same places as with commit_kv; their contents are the quantised rows."""
    rng = np.random.default_rng(6)
    Hkv, dh, N, cap = 2, 8, 9, 12
    Kt, Vt = rng.normal(size=(N, Hkv, dh)), rng.normal(size=(N, Hkv, dh))
    ks, vs = np.array([0.25, 0.75], dtype=np.float32), np.array([1.0, 0.1], dtype=np.float32)
    for start, end, plen, path in [(0, cap, 4, [0, 2, 5]), (3, 9, 4, [0, 1, 4, 7]), (0, cap, 0, [0])]:
        Kc = np.full((cap, Hkv, dh), 0x55, dtype=np.uint8)
        Vc = np.full((cap, Hkv, dh), 0x55, dtype=np.uint8)
        Kw, Vw = np.zeros((cap, Hkv, dh)), np.zeros((cap, Hkv, dh))
        n8 = f8.commit_kv_fp8(Kc, Vc, start, end, plen, Kt, Vt, path, ks, vs)
        n16 = orc.commit_kv(Kw, Vw, start, end, plen, Kt, Vt, path)
        assert n8 == n16
        written = np.any(Kw != 0, axis=(1, 2))
        assert np.all(Kc[~written] == 0x55) and np.all(Vc[~written] == 0x55)
        for t in np.flatnonzero(written):
            assert np.array_equal(Kc[t], f8.quantize_rows(Kw[t], ks))
            assert np.array_equal(Vc[t], f8.quantize_rows(Vw[t], vs))


def test_attention_over_a_dequantised_prefix_stays_close_to_16_bit():
    """A sanity bound that ties the variant to the method: quantising the prefix to 8 bits
    (relative step 2^-4) moves the attention output by a few percent, not more."""
    rng = np.random.default_rng(8)
    Hq, Hkv, dh, P, N = 4, 2, 16, 40, 5
    Q = rng.normal(size=(N, Hq, dh))
    Kp, Vp = rng.normal(size=(P, Hkv, dh)), rng.normal(size=(P, Hkv, dh))
    Kt, Vt = rng.normal(size=(N, Hkv, dh)), rng.normal(size=(N, Hkv, dh))
    mask = np.tril(np.ones((N, N), dtype=bool))
    ks = np.full(Hkv, 2.0 ** -5, dtype=np.float32)
    K8 = f8.dequantize(f8.quantize_rows(Kp, ks), ks)
    V8 = f8.dequantize(f8.quantize_rows(Vp, ks), ks)
    o16, _ = orc.tree_attn(Q, Kp, Vp, Kt, Vt, mask)
    o8, _ = orc.tree_attn(Q, K8, V8, Kt, Vt, mask)
    assert 0 < np.max(np.abs(o8 - o16)) < 0.1
