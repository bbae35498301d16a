"""Pins for the oracle's tree attention (CPU only).

The tree mask of Section 4.2 ("each token can only see its ancestor nodes")
reduces to textbook cases: a chain tree is ordinary causal attention (checked
against torch's scaled_dot_product_attention), a star tree is a two-key softmax
with a closed form, equal value rows make the output independent of the mask,
and attention over a set of keys does not depend on their order.
"""
import numpy as np
import pytest
import torch

from oracle import eagle2_oracle as orc


def _rand(shape, rng):
    return rng.normal(size=shape)


def _chain_mask(n):
    return np.tril(np.ones((n, n), dtype=bool))


@pytest.mark.parametrize("Hq,Hkv,dh,P,N", [(4, 4, 16, 9, 5), (8, 2, 32, 33, 7), (2, 1, 8, 0, 4)])
def test_chain_tree_is_causal_attention(Hq, Hkv, dh, P, N):
    rng = np.random.default_rng(Hq * 100 + P)
    Q, Kp, Vp = _rand((N, Hq, dh), rng), _rand((P, Hkv, dh), rng), _rand((P, Hkv, dh), rng)
    Kt, Vt = _rand((N, Hkv, dh), rng), _rand((N, Hkv, dh), rng)
    O, lse = orc.tree_attn(Q, Kp, Vp, Kt, Vt, _chain_mask(N))
    # library causal attention over the full P+N sequence; the tree rows are its last N rows
    g = Hq // Hkv
    Kf = torch.from_numpy(np.concatenate([Kp, Kt], 0)).repeat_interleave(g, dim=1).permute(1, 0, 2)
    Vf = torch.from_numpy(np.concatenate([Vp, Vt], 0)).repeat_interleave(g, dim=1).permute(1, 0, 2)
    Qf = torch.cat([torch.zeros(P, Hq, dh, dtype=torch.float64), torch.from_numpy(Q)], 0).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(Qf[None], Kf[None], Vf[None], is_causal=True)[0]
    ref = ref.permute(1, 0, 2)[P:].numpy()
    assert np.allclose(O, ref, atol=1e-12, rtol=1e-12)
    # lse against torch.logsumexp of the causal scores
    S = torch.einsum("hqd,hkd->hqk", Qf, Kf) / np.sqrt(dh)
    for i in range(N):
        want = torch.logsumexp(S[:, P + i, : P + i + 1], dim=-1).numpy()
        assert np.allclose(lse[i], want, atol=1e-12)


def test_star_tree_two_key_closed_form():
    """P = 0 and every node a child of the root: row i sees the root and itself, so
    O_i = v_0 + sigmoid(s_ii - s_i0) (v_i - v_0)."""
    rng = np.random.default_rng(2)
    N, H, dh = 6, 3, 8
    Q, Kt, Vt = _rand((N, H, dh), rng), _rand((N, H, dh), rng), _rand((N, H, dh), rng)
    mask = np.eye(N, dtype=bool)
    mask[:, 0] = True
    empty = np.zeros((0, H, dh))
    O, lse = orc.tree_attn(Q, empty, empty, Kt, Vt, mask)
    for h in range(H):
        assert np.allclose(O[0, h], Vt[0, h])
        assert lse[0, h] == pytest.approx(Q[0, h] @ Kt[0, h] / np.sqrt(dh))
        for i in range(1, N):
            s0, si = Q[i, h] @ Kt[0, h] / np.sqrt(dh), Q[i, h] @ Kt[i, h] / np.sqrt(dh)
            w = 1.0 / (1.0 + np.exp(-(si - s0)))
            assert np.allclose(O[i, h], Vt[0, h] + w * (Vt[i, h] - Vt[0, h]), atol=1e-12)
            assert lse[i, h] == pytest.approx(np.logaddexp(s0, si))


def test_equal_values_and_permutation_invariance_and_gqa():
    rng = np.random.default_rng(4)
    N, Hq, Hkv, dh, P = 5, 4, 2, 8, 12
    Q, Kp, Kt = _rand((N, Hq, dh), rng), _rand((P, Hkv, dh), rng), _rand((N, Hkv, dh), rng)
    # a random tree mask: parent of i is a random earlier row
    parent = [-1] + [int(rng.integers(0, i)) for i in range(1, N)]
    mask = np.zeros((N, N), dtype=bool)
    for i in range(N):
        j = i
        while j >= 0:
            mask[i, j] = True
            j = parent[j]
    v = _rand((Hkv, dh), rng)
    O, _ = orc.tree_attn(Q, Kp, np.tile(v, (P, 1, 1)), Kt, np.tile(v, (N, 1, 1)), mask)
    for h in range(Hq):
        assert np.allclose(O[:, h], v[h // (Hq // Hkv)], atol=1e-12)     # GQA head mapping too
    Vp, Vt = _rand((P, Hkv, dh), rng), _rand((N, Hkv, dh), rng)
    O1, l1 = orc.tree_attn(Q, Kp, Vp, Kt, Vt, mask)
    perm = rng.permutation(P)
    O2, l2 = orc.tree_attn(Q, Kp[perm], Vp[perm], Kt, Vt, mask)
    assert np.allclose(O1, O2, atol=1e-12) and np.allclose(l1, l2, atol=1e-12)
    # splitting the prefix: each part also holds the tree keys T, so in the un-normalised
    # domain whole = A + B - T, combined through the log-sum-exps
    cut = 5
    Oa, la = orc.tree_attn(Q, Kp[:cut], Vp[:cut], Kt, Vt, mask)
    Ob, lb = orc.tree_attn(Q, Kp[cut:], Vp[cut:], Kt, Vt, mask)
    Ot, lt = orc.tree_attn(Q, Kp[:0], Vp[:0], Kt, Vt, mask)
    za, zb, zt = np.exp(la), np.exp(lb), np.exp(lt)
    whole = (Oa * za[..., None] + Ob * zb[..., None] - Ot * zt[..., None]) / (za + zb - zt)[..., None]
    assert np.allclose(whole, O1, atol=1e-10)
    assert np.allclose(np.log(za + zb - zt), l1, atol=1e-10)


def test_masked_keys_have_no_influence():
    """Changing the K/V of a tree row that is not an ancestor must not change a row's output."""
    rng = np.random.default_rng(9)
    N, H, dh, P = 4, 2, 8, 3
    Q, Kp, Vp = _rand((N, H, dh), rng), _rand((P, H, dh), rng), _rand((P, H, dh), rng)
    Kt, Vt = _rand((N, H, dh), rng), _rand((N, H, dh), rng)
    mask = np.array([[1, 0, 0, 0], [1, 1, 0, 0], [1, 0, 1, 0], [1, 0, 1, 1]], dtype=bool)
    O1, _ = orc.tree_attn(Q, Kp, Vp, Kt, Vt, mask)
    Kt2, Vt2 = Kt.copy(), Vt.copy()
    Kt2[1] += 5.0
    Vt2[1] -= 3.0                                  # row 1 is a sibling branch of rows 2, 3
    O2, _ = orc.tree_attn(Q, Kp, Vp, Kt2, Vt2, mask)
    assert np.allclose(O1[[0, 2, 3]], O2[[0, 2, 3]], atol=1e-13)
    assert not np.allclose(O1[1], O2[1])
