"""Pins for the oracle's acceptance step (CPU only).

Greedy: brute force over every root-to-node path (the accepted path is the longest
one whose tokens all equal the target's arg-max at their parents).
Sampling: the chain case is exactly the rule of Section 2.1 (re-implemented here
for a plain chain), p == q always accepts, the bonus draw is an inverse CDF, and
the law of the first emitted token equals the target distribution p when the
children are drawn from q without replacement (losslessness, abstract and
Section 2.1) -- computed exactly by enumerating the accept/reject branches.
"""
import itertools

import numpy as np
import pytest

from oracle import eagle2_oracle as orc


def _random_tree(V, hd, D, k, n_tree, seed, scale=2.0):
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, hd))
    st = orc.DraftState(D, k)
    dl = np.zeros((orc.n_draft_rows(D, k), V))
    for d in range(D):
        orc.expand(st, d, rng.normal(size=(1 if d == 0 else k, hd)) * scale, W, draft_logits=dl)
    return st, orc.rerank(st, n_tree, root_token=0, prefix_len=0), dl


def _greedy_bruteforce(tl, tree):
    choice = [int(np.flatnonzero(row == row.max())[0]) for row in tl]
    best = [0]
    for node in range(len(tree.token)):
        path, j = [], node
        while j >= 0:
            path.append(j)
            j = int(tree.parent[j])
        path.reverse()
        ok = all(int(tree.token[path[i]]) == choice[path[i - 1]] for i in range(1, len(path)))
        if ok and len(path) > len(best):
            best = path
    return best, choice[best[-1]]


@pytest.mark.parametrize("seed", range(12))
def test_greedy_is_longest_matching_path(seed):
    V, D, k, N = 6, 4, 3, 14
    st, tree, _ = _random_tree(V, 5, D, k, N, seed)
    rng = np.random.default_rng(100 + seed)
    tl = rng.normal(size=(N, V))
    res = orc.accept_greedy(tl, tree.token, tree.parent)
    path, bonus = _greedy_bruteforce(tl, tree)
    assert res.path == path and res.accept_len == len(path) - 1 and res.bonus_token == bonus


def test_greedy_planted_paths_every_length():
    V, D, k, N = 40, 5, 3, 30
    st, tree, _ = _random_tree(V, 6, D, k, N, seed=7, scale=3.0)
    deepest = int(np.argmax(tree.depth))
    chain = []
    j = deepest
    while j >= 0:
        chain.append(j)
        j = int(tree.parent[j])
    chain.reverse()
    assert len(chain) - 1 >= 3
    for L in range(len(chain)):
        tl = np.zeros((N, V))
        free = [t for t in range(V) if t not in set(tree.token.tolist())][0]
        tl[:, free] = 1.0                               # default: a token no node carries
        for i in range(L):
            tl[chain[i]] = 0.0
            tl[chain[i], tree.token[chain[i + 1]]] = 5.0
        res = orc.accept_greedy(tl, tree.token, tree.parent)
        assert res.accept_len == L and res.path == chain[: L + 1]
        assert res.bonus_token == free
    # arg-max ties go to the lowest token id
    tl = np.zeros((N, V))
    res = orc.accept_greedy(tl, tree.token, tree.parent)
    assert res.bonus_token == 0 or res.accept_len > 0


# ---------------------------------------------------------------------------
# sampling
# ---------------------------------------------------------------------------

def _chain_tree(D, tokens):
    """One child per node, k = 1: candidate ids 0..D-1, draft rows 0..D-1."""
    tree_token = np.array([0] + list(tokens))
    tree_parent = np.arange(-1, D)
    tree_cand = np.arange(-1, D)
    return tree_token, tree_parent, tree_cand


def _textbook_chain(p_rows, q_rows, tokens, ua, ub):
    """Chain speculative sampling as stated in Section 2.1 (front to back)."""
    acc = 0
    for i, x in enumerate(tokens):
        p, q = p_rows[i], q_rows[i]
        if ua[i + 1] < min(1.0, p[x] / q[x]):
            acc += 1
            continue
        r = np.maximum(p - q, 0.0)
        r = r / r.sum()
        return acc, int(np.searchsorted(np.cumsum(r), ub[i] * 1.0, side="right"))
    p = p_rows[len(tokens)]
    return acc, int(np.searchsorted(np.cumsum(p), ub[len(tokens)] * p.sum(), side="right"))


@pytest.mark.parametrize("seed", range(20))
def test_sampling_chain_matches_section_2_1(seed):
    rng = np.random.default_rng(seed)
    V, D, T = 7, 4, 0.7 + 0.1 * (seed % 5)
    tl = rng.normal(size=(D + 1, V)) * 2
    dl = rng.normal(size=(D, V)) * 2
    tokens = rng.integers(0, V, size=D)
    tt, tp, tc = _chain_tree(D, tokens)
    ua, ub = rng.random(D + 1), rng.random(D + 1)
    res = orc.accept_sample(tl, dl, T, ua, ub, tt, tp, tc, topk=1)
    p_rows = [orc.softmax64(tl[i] / T) for i in range(D + 1)]
    q_rows = [orc.softmax64(dl[i]) for i in range(D)]
    acc, bonus = _textbook_chain(p_rows, q_rows, tokens, ua, ub)
    assert (res.accept_len, res.bonus_token) == (acc, bonus)
    assert res.path == list(range(acc + 1))


def test_sampling_identical_distributions_always_accept():
    rng = np.random.default_rng(0)
    V, D = 9, 5
    dl = rng.normal(size=(D, V))
    tl = np.vstack([dl, rng.normal(size=(1, V))])           # p_i == q_i at T = 1
    tokens = rng.integers(0, V, size=D)
    tt, tp, tc = _chain_tree(D, tokens)
    ua = np.full(D + 1, 0.999999)
    res = orc.accept_sample(tl, dl, 1.0, ua, np.zeros(D + 1), tt, tp, tc, topk=1)
    assert res.accept_len == D


def test_bonus_draw_is_inverse_cdf():
    rng = np.random.default_rng(3)
    V = 11
    tl = rng.normal(size=(1, V)) * 2
    p = orc.softmax64(tl[0])
    tt, tp, tc = np.array([0]), np.array([-1]), np.array([-1])
    n = 20000
    counts = np.zeros(V)
    for i in range(n):
        u = (i + 0.5) / n
        res = orc.accept_sample(tl, np.zeros((1, V)), 1.0, np.zeros(1), np.array([u]), tt, tp, tc, topk=3)
        assert res.bonus_token == int(np.searchsorted(np.cumsum(p), u * p.sum(), side="right"))
        counts[res.bonus_token] += 1
    assert np.allclose(counts / n, p, atol=2.0 / n * V)


def _first_token_law(p, q, children, T=1.0):
    """Exact law of the first emitted token for a root with the given ordered
    children, read off the oracle's own accept probabilities and final residual."""
    V = len(p)
    kc = len(children)
    tt = np.array([0] + list(children))
    tp = np.array([-1] + [0] * kc)
    tc = np.array([-1] + list(range(kc)))                  # layer-1 candidates -> draft row 0
    tl = np.vstack([np.log(p)[None] * T, np.zeros((kc, V))])
    dl = np.log(q)[None]
    ua = np.full(kc + 1, 1.0 - 1e-15)                      # reject whenever rejection is possible
    res = orc.accept_sample(tl, dl, T, ua, np.zeros(kc + 1), tt, tp, tc, topk=max(kc, 1))
    law = np.zeros(V)
    alive = 1.0
    for (row, a) in res.trace:
        if row > kc:
            break
        law[children[row - 1]] += alive * a
        alive *= (1.0 - a)
        if a >= 1.0:
            break
    if alive > 0.0 and res.accept_len == 0:
        law += alive * res.final_p
    return law


@pytest.mark.parametrize("seed,kc", [(0, 1), (1, 2), (2, 2), (3, 3), (4, 3), (5, 4)])
def test_sampling_first_token_law_equals_target(seed, kc):
    rng = np.random.default_rng(seed)
    V = 5
    p = orc.softmax64(rng.normal(size=V) * 1.5)
    q = orc.softmax64(rng.normal(size=V) * 1.5)
    total = np.zeros(V)
    mass = 0.0
    for children in itertools.permutations(range(V), kc):
        w, rem = 1.0, 1.0
        for x in children:                                  # drawn from q without replacement
            w *= q[x] / rem
            rem -= q[x]
        total += w * _first_token_law(p, q, list(children))
        mass += w
    assert mass == pytest.approx(1.0, abs=1e-12)
    assert np.allclose(total, p, atol=1e-12)


def test_sampling_follows_tree_and_restarts_at_accepted_child():
    """Two levels: forcing acceptance of the second child of the root must continue
    with that child's own target row and its own children."""
    V, D, k, N = 8, 3, 2, 11                              # all 10 candidates + root
    st, tree, dl = _random_tree(V, 5, D, k, N, seed=21)
    kids0 = [i for i in range(N) if tree.parent[i] == 0]
    assert len(kids0) == 2
    rng = np.random.default_rng(1)
    tl = rng.normal(size=(N, V))
    ua = np.full(N, 1.0 - 1e-15)
    ua[kids0[1]] = 0.0                                     # accept the second sibling
    res = orc.accept_sample(tl, dl, 1.0, ua, np.full(N, 0.5), tree.token, tree.parent, tree.cand, k)
    tested = [row for row, _ in res.trace]
    assert tested[:2] == kids0 and res.path[:2] == [0, kids0[1]]
    grandkids = [i for i in range(N) if tree.parent[i] == kids0[1]]
    assert tested[2:2 + len(grandkids)] == grandkids


# ---------------------------------------------------------------------------
# which draft distribution is q at a node below the root
# ---------------------------------------------------------------------------

def _tree_with_known_rows(seed, V=12, hd=6, D=3, k=3):
    """A full tree (every candidate kept) built with a distinct, test-chosen hidden state per (pass, slot).
    Returns the tree, the dense draft logits as the expansion stored them, and -- built here, without the
    oracle's row helpers -- the distribution each expanded node's children were taken from, keyed by the
    node's candidate id (-1 = root): softmax of that node's own hidden state through the LM head."""
    rng = np.random.default_rng(seed)
    W = rng.normal(size=(V, hd))
    st = orc.DraftState(D, k)
    dl = np.full((orc.n_draft_rows(D, k), V), np.nan)
    q_of = {}
    for d in range(D):
        F = 1 if d == 0 else k
        H = rng.normal(size=(F, hd)) * 2.0
        nodes = [-1] if d == 0 else [int(c) for c in st.frontier[d]]         # who is expanded, slot by slot
        for s, node in enumerate(nodes):
            z = H[s] @ W.T
            e = np.exp(z - z.max())
            q_of[node] = e / e.sum()
        orc.expand(st, d, H, W, draft_logits=dl)
    tree = orc.rerank(st, orc.n_candidates(D, k) + 1, root_token=0, prefix_len=0)
    return st, tree, dl, q_of


@pytest.mark.parametrize("seed", range(8))
def test_sampling_uses_the_distribution_each_parent_was_expanded_with(seed):
    """Section 4.1: a node's children are the top-k of the distribution the draft model produced AT THAT
    NODE; Section 2.1: that distribution is the p-hat of their acceptance test.  Every acceptance ratio the
    oracle reports, at every depth and for expanded nodes in every frontier slot, must be p(x)/q(x) with q
    the distribution the test itself attached to the parent -- including after rejected siblings."""
    V, D, k, T = 12, 3, 3, 0.8
    st, tree, dl, q_of = _tree_with_known_rows(seed)
    N = len(tree.token)
    rng = np.random.default_rng(1000 + seed)
    tl0 = rng.normal(size=(N, V)) * 1.5
    slots_seen = set()
    for steer in itertools.product(range(k), repeat=2):                       # which child to accept at depth 1, 2
        ua = np.full(N, 1.0 - 1e-15)
        tl = tl0.copy()
        cur = 0
        for j in steer:
            kids = [i for i in range(N) if tree.parent[i] == cur]
            if not kids:
                break
            for c in kids[:j]:
                tl[cur, tree.token[c]] = -60.0                                # p(x) ~ 0: certainly rejected
            tl[cur, tree.token[kids[j]]] = 12.0                               # p(x) > q(x) also in the residuals
            cur = kids[j]
            ua[cur] = 0.0                                                     # certainly accepted
        res = orc.accept_sample(tl, dl, T, ua, np.full(N, 0.5), tree.token, tree.parent, tree.cand, k)
        assert res.accept_len >= 2
        checked = 0
        for node in res.path:
            kids = [i for i in range(N) if tree.parent[i] == node]
            cand = int(tree.cand[node])
            if not kids:
                assert cand not in q_of                                        # never expanded: no children, no q
                continue
            z = tl[node] / T
            p = np.exp(z - z.max())
            p /= p.sum()
            q = q_of[cand].copy()
            if cand >= 0:
                d = orc.cand_depth(cand, k)
                slots_seen.add((d, list(st.frontier[d]).index(cand)))
            for c in kids:
                if c not in res.ratios:
                    break                                                     # an earlier sibling was accepted
                x = int(tree.token[c])
                assert res.ratios[c] == pytest.approx(p[x] / q[x], rel=1e-10), (node, c)
                checked += 1
                r = np.maximum(p - q, 0.0)
                p = r / r.sum() if r.sum() > 0 else p
                q[x] = 0.0
                q = q / q.sum()
        assert checked == len(res.ratios) and checked >= 1
    # expanded nodes in slots other than 0 were visited at both depths, so the slot matters
    assert {(1, 1), (1, 2)} <= slots_seen and any(d == 2 and s > 0 for d, s in slots_seen)


def test_draft_rows_of_a_round_are_all_distinct_and_cover_the_matrix():
    """Every (pass, slot) owns one row of the dense draft-logit matrix and the R rows are used exactly once."""
    for D, k in [(1, 4), (3, 3), (6, 10), (8, 16)]:
        rows = [orc.draft_row(d, s, k) for d in range(D) for s in range(1 if d == 0 else k)]
        assert sorted(rows) == list(range(orc.n_draft_rows(D, k)))
