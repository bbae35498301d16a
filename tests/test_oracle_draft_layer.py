"""Pins of the draft-layer oracle against library routines and against the same layer
run causally over a whole sequence with torch ops (an independent formulation).  The
architecture itself is this repository's reading (the paper does not print it)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import draft_layer_oracle as dlo


def _weights(rng, V=40, Hd=16, Hq=4, Hkv=2, dh=8, inter=24):
    r = lambda *s: rng.normal(size=s) * 0.3
    return dlo.DraftWeights(embed=r(V, Hd), fc=r(Hd, 2 * Hd), g_attn=1 + 0.1 * r(Hd), wqkv=r((Hq + 2 * Hkv) * dh, Hd),
                            wo=r(Hd, Hq * dh), g_mlp=1 + 0.1 * r(Hd), wgu=r(2 * inter, Hd), wdown=r(Hd, inter),
                            n_q_heads=Hq, n_kv_heads=Hkv, head_dim=dh, eps=1e-5, rope_theta=10000.0)


def test_rmsnorm_equals_torch():
    rng = np.random.default_rng(0)
    x, g = rng.normal(size=(5, 32)), rng.normal(size=32)
    want = F.rms_norm(torch.from_numpy(x), (32,), torch.from_numpy(g), eps=1e-5).numpy()
    assert np.allclose(dlo.rmsnorm(x, g, 1e-5), want, rtol=1e-12, atol=1e-12)


def test_rope_is_a_complex_rotation_and_preserves_norms():
    rng = np.random.default_rng(1)
    x, pos = rng.normal(size=(6, 3, 16)), np.array([0, 1, 5, 17, 100, 4096])
    got = dlo.rope(x, pos, 10000.0)
    z = x[..., :8] + 1j * x[..., 8:]
    w = np.exp(1j * pos[:, None, None] * (10000.0 ** (-np.arange(8) / 8.0))[None, None, :])
    want = z * w
    assert np.allclose(got[..., :8], want.real, atol=1e-12) and np.allclose(got[..., 8:], want.imag, atol=1e-12)
    assert np.allclose(np.linalg.norm(got, axis=-1), np.linalg.norm(x, axis=-1))
    assert np.array_equal(dlo.rope(x[:1], np.array([0]), 10000.0), x[:1])                  # position 0: identity
    # relative property: <rope(q, m), rope(k, n)> depends on m - n only
    q, k = rng.normal(size=(1, 1, 16)), rng.normal(size=(1, 1, 16))
    d1 = np.sum(dlo.rope(q, np.array([7]), 1e4) * dlo.rope(k, np.array([3]), 1e4))
    d2 = np.sum(dlo.rope(q, np.array([104]), 1e4) * dlo.rope(k, np.array([100]), 1e4))
    assert abs(d1 - d2) < 1e-10


def test_silu_equals_torch():
    x = np.linspace(-8, 8, 101)
    assert np.allclose(dlo.silu(x), F.silu(torch.from_numpy(x)).numpy(), atol=1e-14)


def _torch_causal_layer(w, tokens, prev_feature, P):
    """The same layer over the whole sequence (prefix + chain) with torch library ops."""
    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64))
    T = len(tokens)
    x_in = torch.cat([t(w.embed)[torch.tensor(tokens)], t(prev_feature)], dim=-1)
    x0 = F.linear(x_in, t(w.fc))
    n1 = F.rms_norm(x0, (x0.shape[-1],), t(w.g_attn), eps=w.eps)
    qkv = F.linear(n1, t(w.wqkv))
    Hq, Hkv, dh = w.n_q_heads, w.n_kv_heads, w.head_dim
    q = qkv[:, : Hq * dh].view(T, Hq, dh)
    k = qkv[:, Hq * dh: (Hq + Hkv) * dh].view(T, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].view(T, Hkv, dh)
    pos = torch.arange(T, dtype=torch.float64)
    inv = 10000.0 ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cat([ang.cos(), ang.cos()], -1)[:, None, :], torch.cat([ang.sin(), ang.sin()], -1)[:, None, :]
    rot = lambda u: torch.cat([-u[..., dh // 2:], u[..., : dh // 2]], -1)
    q, k = q * cos + rot(q) * sin, k * cos + rot(k) * sin
    kk, vv = k.repeat_interleave(Hq // Hkv, dim=1), v.repeat_interleave(Hq // Hkv, dim=1)
    o = F.scaled_dot_product_attention(q.transpose(0, 1), kk.transpose(0, 1), vv.transpose(0, 1), is_causal=True)
    h1 = x0 + F.linear(o.transpose(0, 1).reshape(T, Hq * dh), t(w.wo))
    n2 = F.rms_norm(h1, (h1.shape[-1],), t(w.g_mlp), eps=w.eps)
    gu = F.linear(n2, t(w.wgu))
    inter = gu.shape[1] // 2
    y = h1 + F.linear(F.silu(gu[:, :inter]) * gu[:, inter:], t(w.wdown))
    return y.numpy(), k.numpy(), v.numpy()


def test_chain_of_passes_equals_the_causal_layer_over_the_whole_sequence():
    """Prefix of P positions processed in one call, then a chain of single-row passes (what a
    k = 1 draft tree does): features, keys and values equal those of the layer run causally over
    all positions at once with torch's rms_norm / linear / scaled_dot_product_attention / silu."""
    rng = np.random.default_rng(2)
    w = _weights(rng)
    P, D = 5, 4
    T = P + D
    tokens = rng.integers(0, 40, size=T)
    prev = rng.normal(size=(T, 16))
    want_y, want_k, want_v = _torch_causal_layer(w, tokens, prev, P)
    Hkv, dh = w.n_kv_heads, w.head_dim
    # prefix: one call with a causal mask over its own rows, no older prefix
    Kt, Vt = np.zeros((P, Hkv, dh)), np.zeros((P, Hkv, dh))
    y_pre = dlo.draft_layer(w, tokens[:P], prev[:P], np.arange(P), np.zeros((0, Hkv, dh)), np.zeros((0, Hkv, dh)),
                            Kt, Vt, list(range(P)), np.tril(np.ones((P, P), dtype=bool)))
    assert np.allclose(y_pre, want_y[:P], atol=1e-10) and np.allclose(Kt, want_k[:P], atol=1e-10)
    # chain: pass d sees the prefix and tree rows 0..d
    Ktree, Vtree = np.zeros((D, Hkv, dh)), np.zeros((D, Hkv, dh))
    for d in range(D):
        mask = np.zeros((1, D), dtype=bool)
        mask[0, : d + 1] = True
        y = dlo.draft_layer(w, tokens[P + d: P + d + 1], prev[P + d: P + d + 1], np.array([P + d]), Kt, Vt,
                            Ktree, Vtree, [d], mask)
        assert np.allclose(y[0], want_y[P + d], atol=1e-10), f"pass {d}"
    assert np.allclose(Ktree, want_k[P:], atol=1e-10) and np.allclose(Vtree, want_v[P:], atol=1e-10)


def test_siblings_do_not_see_each_other():
    """Two rows of one pass with the same inputs get the same feature whatever the other row is
    (ancestor-only visibility, Section 4.1)."""
    rng = np.random.default_rng(3)
    w = _weights(rng)
    Hkv, dh = w.n_kv_heads, w.head_dim
    Kp, Vp = rng.normal(size=(3, Hkv, dh)), rng.normal(size=(3, Hkv, dh))
    prev = rng.normal(size=(2, 16))
    out = []
    for other in (7, 23):
        Kt, Vt = np.zeros((2, Hkv, dh)), np.zeros((2, Hkv, dh))
        y = dlo.draft_layer(w, np.array([5, other]), prev, np.array([3, 3]), Kp, Vp, Kt, Vt, [0, 1], np.eye(2, dtype=bool))
        out.append(y[0])
    assert np.array_equal(out[0], out[1])
