"""Pins for the oracle's expansion, reranking and flattening (CPU only).

Each test checks the oracle against something other than itself: the paper's
stated invariants (Section 4.2), brute-force enumeration of every path, a closed
form for a context-free draft model, library routines (log_softmax + topk) for
the degenerate shapes, and the hyper-parameters the paper prints (Appendix A).
"""
import heapq
import itertools
import json
import os

import numpy as np
import pytest
import torch
from scipy.special import log_softmax as scipy_log_softmax

from oracle import eagle2_oracle as orc


def _path_of(state, cid):
    toks = []
    while cid >= 0:
        toks.append(int(state.token[cid]))
        cid = int(state.parent[cid])
    return tuple(reversed(toks))


def _hidden_of_path(path, hd, seed):
    """A hidden state that depends on the whole token path (context dependence)."""
    h = abs(hash((seed,) + tuple(path))) % (2 ** 32)
    return np.random.default_rng(h).normal(0.0, 1.5, size=hd)


def _run_path_model(V, hd, D, k, seed):
    rng = np.random.default_rng(seed)
    W = rng.normal(0.0, 1.0, size=(V, hd))
    st = orc.DraftState(D, k)
    for d in range(D):
        if d == 0:
            H = _hidden_of_path((), hd, seed)[None, :]
        else:
            H = np.stack([_hidden_of_path(_path_of(st, int(c)), hd, seed) for c in st.frontier[d]])
        orc.expand(st, d, H, W)
    return W, st


# ---------------------------------------------------------------------------
# P2: brute force over every path, tiny vocabularies
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("V,D,k,seed", [(5, 3, 2, 1), (6, 3, 3, 2), (4, 3, 2, 3), (6, 2, 3, 4), (5, 3, 3, 5)])
def test_bruteforce_all_paths(V, D, k, seed):
    hd = 6
    W, st = _run_path_model(V, hd, D, k, seed)

    # independent joint log-probability of every path up to length D
    joint = {}
    for L in range(1, D + 1):
        for path in itertools.product(range(V), repeat=L):
            lp = 0.0
            for i in range(L):
                logits = W @ _hidden_of_path(path[:i], hd, seed)
                lp += scipy_log_softmax(logits)[path[i]]
            joint[path] = lp

    def topk_tokens(prefix):
        lp = scipy_log_softmax(W @ _hidden_of_path(prefix, hd, seed))
        return sorted(range(V), key=lambda t: (-lp[t], t))[:k]

    # declarative layers: a node exists iff its parent was in the previous frontier and
    # its token is among the parent's k most probable; a frontier is the k best of a layer
    layers, frontier = {}, {0: [()]}
    for L in range(1, D + 1):
        nodes = [p + (t,) for p in frontier[L - 1] for t in topk_tokens(p)]
        layers[L] = nodes
        frontier[L] = sorted(nodes, key=lambda p: -joint[p])[:k]

    # the oracle's candidates, layer by layer
    got_paths = {}
    for cid in range(orc.n_candidates(D, k)):
        got_paths[_path_of(st, cid)] = float(st.score[cid])
    want_paths = {p for L in layers for p in layers[L]}
    assert set(got_paths) == want_paths
    for p, s in got_paths.items():
        assert s == pytest.approx(joint[p], abs=1e-12)
    for L in range(1, D):
        got = {_path_of(st, int(c)) for c in st.frontier[L]}
        assert got == set(frontier[L])
        # and the frontier is ordered by decreasing value
        vals = [joint[_path_of(st, int(c))] for c in st.frontier[L]]
        assert vals == sorted(vals, reverse=True)

    # rerank: the m best of *all* nodes
    for m in range(1, len(want_paths) + 1):
        tree = orc.rerank(st, m + 1, root_token=0, prefix_len=0)
        got = {_path_of(st, int(c)) for c in tree.cand[1:]}
        want = set(sorted(want_paths, key=lambda p: -joint[p])[:m])
        assert got == want


# ---------------------------------------------------------------------------
# P3: closed form for a context-free draft model; the shallower-first tie rule
# ---------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_context_free_product_tree(seed):
    """Same hidden state everywhere => every node has the same child distribution c,
    and a path's value is the sum of log c over its tokens.  For m <= k the selected
    values must be the m largest over the *unconstrained* product tree (a node in the
    global top-m has its whole ancestry in the top-m, hence in every frontier)."""
    V, hd, D, k = 12, 5, 4, 4
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, hd))
    h = rng.normal(size=hd) * 2.0
    st = orc.DraftState(D, k)
    for d in range(D):
        orc.expand(st, d, np.tile(h, (1 if d == 0 else k, 1)), W)
    c = scipy_log_softmax(W @ h)
    best_tokens = np.sort(c)[::-1][:k]
    # best-first enumeration over multisets of token log-probs (order-free values)
    heap = [(-v, (i,)) for i, v in enumerate(best_tokens)]
    heapq.heapify(heap)
    want = []
    while heap and len(want) < k:
        negv, idx = heapq.heappop(heap)
        want.append(-negv)
        if len(idx) < D:
            for j in range(k):
                heapq.heappush(heap, (negv - best_tokens[j], idx + (j,)))
    for m in range(1, k + 1):
        tree = orc.rerank(st, m + 1, 7, 0)
        got = sorted((float(st.score[int(cid)]) for cid in tree.cand[1:]), reverse=True)
        assert got == pytest.approx(want[:m], abs=1e-12)


def test_equal_values_prefer_shallower():
    """Rows whose best token has probability exactly 1 give a chain of nodes that
    all have value exactly 0 (log 1); the paper's rule selects the shallower ones."""
    V, D, k = 5, 3, 2
    W = np.zeros((V, 2))
    W[0, 0] = 1.0
    W[1:, 0] = -1.0
    h = np.array([1.0e4, 0.0])       # logits: [1e4, -1e4, ...] -> softmax = one-hot exactly
    st = orc.DraftState(D, k)
    for d in range(D):
        lp = orc.expand(st, d, np.tile(h, (1 if d == 0 else k, 1)), W)
        assert lp[0, 0] == 0.0
    zero_nodes = [c for c in range(orc.n_candidates(D, k)) if st.score[c] == 0.0]
    assert [orc.cand_depth(c, k) for c in zero_nodes] == [1, 2, 3]
    for m in (1, 2, 3):
        tree = orc.rerank(st, m + 1, 0, 0)
        assert list(tree.depth[1:]) == list(range(1, m + 1))
        assert list(tree.parent) == [-1] + list(range(m))


# ---------------------------------------------------------------------------
# P4: degenerate shapes reduce to library routines
# ---------------------------------------------------------------------------

def test_depth_one_is_library_topk():
    V, hd, k = 300, 16, 8
    rng = np.random.default_rng(11)
    W, h = rng.normal(size=(V, hd)), rng.normal(size=(1, hd))
    st = orc.DraftState(1, k)
    orc.expand(st, 0, h, W)
    lp = torch.log_softmax(torch.from_numpy(h @ W.T)[0], dim=0)
    vals, idx = torch.topk(lp, k)
    assert list(st.token) == idx.tolist()
    assert np.allclose(st.score, vals.numpy(), atol=1e-12)
    tree = orc.rerank(st, 6, 42, 10)
    assert list(tree.token) == [42] + sorted_by_cand(idx.tolist()[:5])
    assert list(tree.position) == [10] + [11] * 5


def sorted_by_cand(tokens_in_rank_order):
    # candidates of layer 1 are numbered in rank order, and the flat order is by id
    return list(tokens_in_rank_order)


def test_topk_one_is_greedy_chain():
    V, hd, D = 50, 8, 5
    rng = np.random.default_rng(5)
    W = rng.normal(size=(V, hd))
    Hs = rng.normal(size=(D, hd)) * 2
    st = orc.DraftState(D, 1)
    total = 0.0
    for d in range(D):
        orc.expand(st, d, Hs[d][None], W)
        lp = torch.log_softmax(torch.from_numpy(W @ Hs[d]), dim=0)
        total += float(lp.max())
        assert int(st.token[d]) == int(lp.argmax())
        assert float(st.score[d]) == pytest.approx(total, abs=1e-12)
        assert int(st.parent[d]) == d - 1
    tree = orc.rerank(st, D + 1, 3, 100)
    assert list(tree.parent) == list(range(-1, D))
    assert np.array_equal(tree.mask, np.tril(np.ones((D + 1, D + 1), dtype=bool)))  # chain = lower triangular
    assert list(tree.position) == list(range(100, 100 + D + 1))


# ---------------------------------------------------------------------------
# P1 + P5: the paper's invariants at the paper's hyper-parameters
# ---------------------------------------------------------------------------

def _golden():
    with open(os.path.join(os.path.dirname(__file__), "golden", "paper_constants.json")) as f:
        return json.load(f)


def _random_round(V, hd, D, k, seed, scale):
    rng = np.random.default_rng(seed)
    W = rng.normal(0, 0.3, size=(V, hd))
    st = orc.DraftState(D, k)
    for d in range(D):
        F = 1 if d == 0 else k
        orc.expand(st, d, rng.normal(0, scale, size=(F, hd)), W)
    return st


@pytest.mark.parametrize("model", ["7b_8b", "13b", "70b"])
@pytest.mark.parametrize("scale", [0.5, 3.0])
def test_paper_hyperparameters_and_invariants(model, scale):
    g = _golden()["eagle2"]
    D, k, m = g["depth"], g["expand_nodes"], g["total_draft_tokens"][model]
    assert (D, k) == (6, 10)
    st = _random_round(400, 24, D, k, seed=m, scale=scale)
    C = orc.n_candidates(D, k)
    assert C == 510 and orc.n_draft_rows(D, k) == 51
    # value of a node never exceeds its parent's (Section 4.2)
    for c in range(C):
        p = int(st.parent[c])
        assert st.score[c] <= (0.0 if p < 0 else st.score[p])
        assert orc.cand_depth(c, k) == (1 if p < 0 else orc.cand_depth(p, k) + 1)
    # siblings are distinct tokens; each frontier is a subset of its layer
    for d in range(D):
        F = 1 if d == 0 else k
        base = orc.cand_base(d, k)
        for s in range(F):
            sib = st.token[base + s * k: base + (s + 1) * k]
            assert len(set(sib.tolist())) == k
        if d + 1 < D:
            assert all(base <= c < base + F * k for c in st.frontier[d + 1])
    tree = orc.rerank(st, m, root_token=1, prefix_len=77)
    N = m
    assert tree.token.shape == (N,)                      # exactly the configured total
    sel = set(int(c) for c in tree.cand[1:])
    assert len(sel) == N - 1
    for c in sel:                                        # connected tree (Section 4.2)
        assert int(st.parent[c]) == -1 or int(st.parent[c]) in sel
    worst_in = min(st.score[list(sel)])
    best_out = max(st.score[c] for c in range(C) if c not in sel)
    assert worst_in >= best_out
    for i in range(N):
        assert tree.mask[i].sum() == tree.depth[i] + 1   # self + ancestors incl. root
        assert tree.position[i] == 77 + tree.depth[i]
        if i:
            par = int(tree.parent[i])
            assert par < i
            want = tree.mask[par].copy()
            want[i] = True
            assert np.array_equal(tree.mask[i], want)
        for j in range(N):
            bit = (int(tree.mask_bits[i, j // 64]) >> (j % 64)) & 1
            assert bit == int(tree.mask[i, j])


def test_figure_toy_shape():
    """The method figure's setting (expand 2 nodes per layer, keep 8): shapes only,
    the node values printed inside the figure are not part of the text."""
    g = _golden()["figure_toy"]
    k, m = g["expand_nodes"], g["rerank_keep"]
    st = _random_round(20, 8, 3, k, seed=0, scale=2.0)
    tree = orc.rerank(st, m + 1, 0, 0)
    assert tree.token.shape[0] == m + 1 and orc.n_candidates(3, k) == 2 + 2 * 4


def test_ablation_switches():
    """Section 5.2: without reranking the draft is the union of the frontiers;
    without value the frontier is ranked by the node's own confidence."""
    D, k = 4, 3
    rng = np.random.default_rng(3)
    W = rng.normal(size=(30, 6))
    Hs = [rng.normal(size=(1 if d == 0 else k, 6)) * 2 for d in range(D)]
    a, b = orc.DraftState(D, k), orc.DraftState(D, k)
    for d in range(D):
        orc.expand(a, d, Hs[d], W)
        lp = orc.expand(b, d, Hs[d], W, rank_by_value=False)
        if 0 < d < D - 1:
            base = orc.cand_base(d, k)
            own = np.array([lp[(c - base) // k, b.token[c]] for c in range(base, base + k * k)])
            want = set((base + np.argsort(-own)[:k]).tolist())
            assert set(b.frontier[d + 1].tolist()) == want
    t = orc.rerank(a, 0, 0, 0, use_rerank=False)
    last = list(range(orc.cand_base(D - 1, k), orc.n_candidates(D, k)))
    last_best = sorted(last, key=lambda c: -a.score[c])[:k]
    assert set(t.cand[1:].tolist()) == set(a.frontier[1:].reshape(-1).tolist()) | set(last_best)


def test_ablation_closed_forms_context_free():
    """Section 5.2 on a context-free draft (every row has the same distribution c_1 > c_2 > ...),
    where both ablated selections have closed forms that differ from the full method's.
    Ranked by confidence, the k rank-0 children (one per parent) tie at c_1 and win in parent
    order; ranked by value, slot 0's children compete with their parent's head start.
    Without reranking the tree has exactly k nodes per layer."""
    D, k, V = 4, 3, 12
    x = np.linspace(2.0, -3.0, V)                      # strictly decreasing logits: token v has rank v
    W = np.eye(V)
    H = [np.tile(x, (1 if d == 0 else k, 1)) for d in range(D)]
    lp = x - np.log(np.sum(np.exp(x)))
    conf, val = orc.DraftState(D, k), orc.DraftState(D, k)
    for d in range(D):
        orc.expand(conf, d, H[d], W, rank_by_value=False)
        orc.expand(val, d, H[d], W)
    for d in range(2, D):
        base = orc.cand_base(d - 1, k)
        assert conf.frontier[d].tolist() == [base + s * k for s in range(k)]       # rank-0 child of every slot
        assert np.allclose(conf.own[conf.frontier[d]], lp[0])
    # by value the best path keeps winning: frontier 2 = children 0, 1 of slot 0 and child 0 of slot 1
    # iff 2*lp[0] > lp[0]+lp[1] > max(lp[1]+lp[0] (tie, higher id), lp[0]+lp[2])
    assert val.frontier[2].tolist() == [orc.cand_base(1, k), orc.cand_base(1, k) + 1, orc.cand_base(1, k) + k]
    # w/o reranking: k nodes per layer, D*k + 1 rows; last layer by confidence = rank-0 children again
    t_both = orc.rerank(conf, D * k + 1, 0, 0, use_rerank=False, rank_by_value=False)
    assert np.bincount(t_both.depth).tolist() == [1] + [k] * D
    lastb = orc.cand_base(D - 1, k)
    assert t_both.cand[-k:].tolist() == [lastb + s * k for s in range(k)]
    t_val = orc.rerank(val, D * k + 1, 0, 0, use_rerank=False)
    assert np.bincount(t_val.depth).tolist() == [1] + [k] * D
    best_last = sorted(range(lastb, orc.n_candidates(D, k)), key=lambda c: (-val.score[c], c))[:k]
    assert sorted(t_val.cand[-k:].tolist()) == sorted(best_last)
    # value of every node is the sum of its path's confidences (value equation, Section 4.1)
    for st in (conf, val):
        for c in range(orc.n_candidates(D, k)):
            if st.parent[c] >= 0:
                assert abs(st.score[c] - (st.score[st.parent[c]] + st.own[c])) < 1e-12


def test_static_shape_special_cases():
    """Section 2.2: a fixed shape filled in by the drafting phase.  Two shapes have known answers:
    the full k-ary tree equals the dynamic tree that keeps every candidate, and the rank-0 chain
    equals greedy chain decoding (the k = 1 dynamic tree)."""
    rng = np.random.default_rng(8)
    V, Hd, D, k = 25, 6, 3, 3
    W = rng.normal(size=(V, Hd))
    Hs = [rng.normal(size=(1 if d == 0 else k, Hd)) * 2 for d in range(D)]
    # full 3-ary tree of depth 2 inside a D = 2 round: every candidate is a node
    nodes = [(-1, r) for r in range(k)] + [(p, r) for p in range(k) for r in range(k)]
    ids, front = orc.static_shape(nodes, 2, k)
    assert sorted(ids.tolist()) == list(range(orc.n_candidates(2, k))) and front[1].tolist() == [0, 1, 2]
    a, b = orc.DraftState(2, k), orc.DraftState(2, k)
    for d in range(2):
        orc.expand(a, d, Hs[d], W, static_frontier=front[d + 1] if d + 1 < 2 else None)
        orc.expand(b, d, Hs[d], W)
    ta = orc.rerank(a, len(ids) + 1, 0, 0, static_sel=np.sort(ids))
    tb = orc.rerank(b, orc.n_candidates(2, k) + 1, 0, 0)
    assert np.array_equal(ta.token, tb.token) and np.array_equal(ta.parent, tb.parent) and np.array_equal(ta.mask, tb.mask)
    # rank-0 chain of depth 3: slot 0 only; equals the k = 1 dynamic tree on slot 0's hidden states
    ids, front = orc.static_shape([(-1, 0), (0, 0), (1, 0)], D, k)
    assert ids.tolist() == [0, orc.cand_base(1, k), orc.cand_base(2, k)] and front[:, 0].tolist() == [-1, 0, orc.cand_base(1, k)]
    c, g = orc.DraftState(D, k), orc.DraftState(D, 1)
    for d in range(D):
        orc.expand(c, d, Hs[d], W, static_frontier=front[d + 1] if d + 1 < D else None)
        orc.expand(g, d, Hs[d][:1], W)
    tc = orc.rerank(c, D + 1, 0, 0, static_sel=ids)
    tg = orc.rerank(g, D + 1, 0, 0)
    assert np.array_equal(tc.token, tg.token) and np.array_equal(tc.parent, tg.parent) and np.array_equal(tc.depth, tg.depth)
    assert np.all(np.isneginf(c.score[orc.cand_base(1, k) + k: orc.cand_base(2, k)]))      # unused slots stay empty
