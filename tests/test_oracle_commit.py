"""Pins of the oracle's commit step: several rounds chained through it.

The external facts used: at temperature 0 the method is lossless (Section 5: the
generated text equals vanilla decoding), whatever the draft proposes; and a KV cache
grown round by round is the same prefix as the keys of the committed text.
"""
import numpy as np
import pytest

from oracle import eagle2_oracle as orc


def _toy_round(rng, g, root, D, k, n_tree, V, draft_quality):
    """One round on a toy target whose next token depends on the last token only (table g).
    The draft sees a noisy version of the same table, so some branches are right."""
    st = orc.DraftState(D, k)
    W = np.eye(V)
    for d in range(D):
        toks = [root] if d == 0 else [int(st.token[c]) for c in st.frontier[d]]
        H = rng.normal(size=(len(toks), V))
        for s, t in enumerate(toks):
            H[s, g[t]] += draft_quality
        orc.expand(st, d, H, W)
    tree = orc.rerank(st, n_tree, root, 0)
    tl = rng.normal(size=(n_tree, V))
    for i in range(n_tree):
        tl[i, g[int(tree.token[i])]] += 20.0
    return tree, orc.accept_greedy(tl, tree.token, tree.parent)


@pytest.mark.parametrize("quality", [0.0, 2.0, 6.0])
def test_multi_round_greedy_equals_vanilla_decoding(quality):
    rng = np.random.default_rng(11)
    V, D, k, n_tree = 17, 4, 3, 14
    g = rng.permutation(V)
    start = 5
    want = [start]
    while len(want) < 60:
        want.append(int(g[want[-1]]))
    text, root, plen, lens = [start], start, 0, []
    while len(text) < 40:
        tree, res = _toy_round(rng, g, root, D, k, n_tree, V, quality)
        out = orc.commit_round(tree.token, res.path, res.bonus_token, plen)
        assert len(out.tokens) == res.accept_len + 1 and out.prefix_len == plen + res.accept_len + 1
        text += out.tokens
        root, plen = out.root_token, out.prefix_len
        lens.append(res.accept_len)
    assert text == want[: len(text)]
    assert plen == len(text) - 1                   # every token but the pending root has a KV row
    if quality >= 6.0:
        assert max(lens) == D                      # good drafts are accepted to full depth
    if quality == 0.0:
        assert min(lens) == 0


def test_committed_cache_is_the_concatenated_prefix():
    """Attention of the next round over the cache grown by commit_kv equals attention over
    prefix + accepted rows written out by hand; rejected rows leave no trace."""
    rng = np.random.default_rng(5)
    Hkv, dh, P, N, cap = 2, 8, 6, 9, 16
    start = 3                                      # region [3, 3 + cap) of a larger buffer
    Kc, Vc = np.full((40, Hkv, dh), np.nan), np.full((40, Hkv, dh), np.nan)
    Kc[start:start + P], Vc[start:start + P] = rng.normal(size=(P, Hkv, dh)), rng.normal(size=(P, Hkv, dh))
    Kt, Vt = rng.normal(size=(N, Hkv, dh)), rng.normal(size=(N, Hkv, dh))
    before = Kc.copy()
    path = [0, 2, 5, 8]
    n = orc.commit_kv(Kc, Vc, start, start + cap, P, Kt, Vt, path)
    assert n == P + len(path)
    assert np.array_equal(Kc[start + P:start + n], Kt[path]) and np.array_equal(Vc[start + P:start + n], Vt[path])
    untouched = np.ones(40, dtype=bool)
    untouched[start + P:start + n] = False
    assert np.array_equal(np.isnan(Kc[untouched]), np.isnan(before[untouched]))
    assert np.array_equal(Kc[start:start + P], before[start:start + P])
    # next round: a 3-row chain attends over the grown cache
    Q = rng.normal(size=(3, 4, dh))
    K2, V2 = rng.normal(size=(3, Hkv, dh)), rng.normal(size=(3, Hkv, dh))
    mask = np.tril(np.ones((3, 3), dtype=bool))
    got, _ = orc.tree_attn(Q, Kc[start:start + n], Vc[start:start + n], K2, V2, mask)
    by_hand_K = np.concatenate([before[start:start + P], Kt[[0]], Kt[[2]], Kt[[5]], Kt[[8]]])
    by_hand_V = np.concatenate([Vc[start:start + P], Vt[[0]], Vt[[2]], Vt[[5]], Vt[[8]]])
    want, _ = orc.tree_attn(Q, by_hand_K, by_hand_V, K2, V2, mask)
    assert np.array_equal(got, want)


def test_commit_drops_rows_beyond_the_region():
    Kc, Vc = np.zeros((10, 1, 2)), np.zeros((10, 1, 2))
    Kt, Vt = np.arange(8.0).reshape(4, 1, 2) + 1, -np.arange(8.0).reshape(4, 1, 2) - 1
    n = orc.commit_kv(Kc, Vc, 2, 6, 2, Kt, Vt, [0, 1, 3])         # room for two more rows only
    assert n == 4 and np.array_equal(Kc[4:6], Kt[[0, 1]]) and not Kc[6:].any() and not Kc[:4].any()


def test_commit_round_hidden_and_tokens():
    tok = np.array([9, 4, 7, 1, 3])
    hid = np.arange(15.0).reshape(5, 3)
    out = orc.commit_round(tok, [0, 2, 3], 6, 100, hid)
    assert out.tokens == [7, 1, 6] and out.root_token == 6 and out.prefix_len == 103
    assert np.array_equal(out.next_hidden, hid[3])
    out0 = orc.commit_round(tok, [0], 2, 7, hid)
    assert out0.tokens == [2] and out0.prefix_len == 8 and np.array_equal(out0.next_hidden, hid[0])
