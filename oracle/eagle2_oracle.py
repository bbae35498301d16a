"""CPU oracle for one draft-plus-verify round of the context-aware dynamic draft tree.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain reference that the HIP
path is compared against.  It is imported by the tests, by the smoke check and
by the benchmark's cpu-baseline leg, and by nothing in the product path.  It
shares no code with the HIP library and never calls it.

Everything is computed in float64 with numpy, one sequence at a time, following
the paper's steps in the paper's order:

  expand      Section 4.1 (expansion phase) and its value equation
              V_i = prod_{t_j in Path(root, t_i)} c_j, kept as a sum of logs
  rerank      Section 4.2, first paragraph (top-m of all draft tokens, ties to
              the shallower node)
  flatten     Section 4.2, second paragraph (1-D sequence, ancestor-only mask)
  tree_attn   Section 4.2, second paragraph (each token sees its ancestors) on
              top of ordinary attention over the preceding tokens
  accept_*    Section 2.1 (front-to-back acceptance with min(1, p/p_hat), residual
              norm(max(0, p - p_hat))) and Section 2.2 ("Verification Stage":
              alternative branches are attempted after a rejection)
  commit_*    Section 2.1 (accepted tokens are kept, the rest of the draft is
              discarded) on a pre-allocated KV cache (Appendix, "Implementation
              Details"): what one round leaves behind for the next

Conventions (readings of points the paper leaves open; listed in the design
notes of this repository):
  * Pass d (0-based) turns the layer-d frontier into layer d+1.  Pass 0 has one
    row (the root); later passes have k rows.
  * Candidate ids are assigned in generation order: layer 1 gets 0..k-1, layer
    L>=2 gets k + (L-2) k^2 + slot*k + rank.  A larger id is never shallower, so
    "lower id first" realises the paper's "shallower first" tie rule.
  * The flattened tree has n_tree rows: row 0 is the root, then the selected
    candidates in increasing id order.

Pinning status: expand/rerank/flatten, tree_attn and accept_greedy are pinned by
tests/test_oracle_*.py against brute force, closed forms, library routines and
the invariants the paper states.  accept_sample is pinned for the chain case
(Section 2.1's rule) and by the exactness of the emitted-token law; which draft
distribution is q at a node (the one its parent was expanded with, Section 4.1;
draft_row / parent_draft_row) is pinned on full trees whose every expanded node
carries a distribution chosen by the test; the order in
which sibling branches are tried and the renormalisation of the draft
distribution after a rejected sibling are this repository's reading of Section
2.2 -- "parity unpinned" by the paper for that particular choice.  commit_* is
pinned by multi-round decoding: the emitted stream equals vanilla greedy
decoding, and attention over the committed cache equals attention over an
explicitly concatenated prefix.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np


# ----------------------------------------------------------------------------
# index helpers
# ----------------------------------------------------------------------------

def n_candidates(depth: int, topk: int) -> int:
    """C: nodes produced by `depth` passes (k from the root, then k*k per pass)."""
    return topk + (depth - 1) * topk * topk


def n_draft_rows(depth: int, topk: int) -> int:
    """R: LM-head rows evaluated in a round (1 for the root, k per later pass)."""
    return 1 + (depth - 1) * topk


def cand_base(d: int, topk: int) -> int:
    """First candidate id produced by pass d."""
    return 0 if d == 0 else topk + (d - 1) * topk * topk


def cand_depth(cid: int, topk: int) -> int:
    """Tree layer (root = 0) of candidate `cid`."""
    return 1 if cid < topk else 2 + (cid - topk) // (topk * topk)


def draft_row(d: int, slot: int, topk: int) -> int:
    """Row of the per-round draft-logit matrix written by pass d for frontier slot `slot`."""
    return 0 if d == 0 else 1 + (d - 1) * topk + slot


def parent_draft_row(child_cid: int, topk: int) -> int:
    """Draft-logit row of the pass that produced candidate `child_cid`
    (i.e. the distribution its parent was expanded with)."""
    layer = cand_depth(child_cid, topk)
    if layer == 1:
        return 0
    slot = ((child_cid - topk) % (topk * topk)) // topk
    return draft_row(layer - 1, slot, topk)


def log_softmax64(x: np.ndarray) -> np.ndarray:
    """log of the softmax of a vector: x - max - log(sum(exp(x - max)))."""
    x = np.asarray(x, dtype=np.float64)
    m = np.max(x)
    return x - m - np.log(np.sum(np.exp(x - m)))


def softmax64(x: np.ndarray) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    e = np.exp(x - np.max(x))
    return e / np.sum(e)


# ----------------------------------------------------------------------------
# draft state
# ----------------------------------------------------------------------------

@dataclass
class DraftState:
    """Candidate arrays of one sequence's draft tree while it is being expanded."""
    depth: int
    topk: int
    token: np.ndarray = field(init=False)      # [C] token id of each candidate
    score: np.ndarray = field(init=False)      # [C] sum of log confidences along the root path
    parent: np.ndarray = field(init=False)     # [C] candidate id of the parent, -1 = root
    frontier: np.ndarray = field(init=False)   # [D, k] candidate ids expanded by pass d (row 0 unused)
    own: np.ndarray = field(init=False)        # [C] each candidate's own log confidence (score minus the parent's)

    def __post_init__(self):
        c = n_candidates(self.depth, self.topk)
        self.token = np.full(c, -1, dtype=np.int64)
        self.score = np.full(c, -np.inf, dtype=np.float64)
        self.parent = np.full(c, -1, dtype=np.int64)
        self.frontier = np.full((self.depth, self.topk), -1, dtype=np.int64)
        self.own = np.full(c, -np.inf, dtype=np.float64)

    def copy(self) -> "DraftState":
        s = DraftState(self.depth, self.topk)
        s.token, s.score = self.token.copy(), self.score.copy()
        s.parent, s.frontier = self.parent.copy(), self.frontier.copy()
        s.own = self.own.copy()
        return s


# ----------------------------------------------------------------------------
# expansion phase (Section 4.1)
# ----------------------------------------------------------------------------

def expand(state: DraftState, d: int, H, W, draft_logits: Optional[np.ndarray] = None,
           rank_by_value: bool = True, static_frontier: Optional[np.ndarray] = None) -> np.ndarray:
    """One expansion pass.

    H [F, Hd] are the hidden states of the layer-d frontier (F = 1 at d = 0, else
    k; row s belongs to frontier slot s), W [V, Hd] is the LM head.  Each row's
    token distribution is softmax(H W^T) (the draft model's confidence, Section
    3.2); its k most probable tokens become children whose value is the parent's
    value times the confidence (value equation of Section 4.1; kept in logs).
    The k new nodes of highest value form the next frontier (Section 4.1, last
    paragraph).  Returns the [F, V] log-probabilities.

    rank_by_value=False is the "w/o value" ablation of Section 5.2: the next
    frontier is ranked by the nodes' own confidence instead of the path product.

    static_frontier [k] (candidate ids, -1 = unused slot) is the fixed-shape tree the
    method replaces (Section 2.2, differences between EAGLE and EAGLE-2): the nodes
    expanded next are given by the shape instead of being selected; rows of unused
    slots of the current frontier are skipped.
    """
    k, D = state.topk, state.depth
    Hm = np.asarray(H, dtype=np.float64)
    Wm = np.asarray(W, dtype=np.float64)
    F = 1 if d == 0 else k
    Hm = Hm.reshape(-1, Hm.shape[-1])[:F]
    V = Wm.shape[0]
    x = Hm @ Wm.T                                            # [F, V] logits
    logp = np.empty_like(x)
    base = cand_base(d, k)
    tok_ids = np.arange(V)
    for s in range(F):
        logp[s] = log_softmax64(x[s])
        if draft_logits is not None:
            draft_logits[draft_row(d, s, k)] = x[s]
        best = np.lexsort((tok_ids, -logp[s]))[:k]           # most probable first, ties to the lower id
        par = -1 if d == 0 else int(state.frontier[d, s])
        if d > 0 and par < 0:
            continue                                         # unused slot of a fixed shape
        par_score = 0.0 if d == 0 else float(state.score[par])
        for r, v in enumerate(best):
            cid = base + s * k + r
            state.token[cid] = v
            state.score[cid] = par_score + logp[s, v]
            state.parent[cid] = par
            state.own[cid] = logp[s, v]
    if d + 1 < D:
        if static_frontier is not None:
            state.frontier[d + 1] = np.asarray(static_frontier, dtype=np.int64)
        else:
            new = np.arange(base, base + F * k)
            key = state.score[new] if rank_by_value else state.own[new]
            order = np.lexsort((new, -key))[:k]
            state.frontier[d + 1] = new[order]
    return logp


# ----------------------------------------------------------------------------
# reranking phase and flattening (Section 4.2)
# ----------------------------------------------------------------------------

@dataclass
class FlatTree:
    token: np.ndarray        # [N] token ids, row 0 = root token
    parent: np.ndarray       # [N] flat row of the parent, -1 for the root
    depth: np.ndarray        # [N]
    cand: np.ndarray         # [N] candidate id of the row, -1 for the root
    position: np.ndarray     # [N] prefix_len + depth
    mask: np.ndarray         # [N, N] bool: mask[i, j] = j is i or an ancestor of i
    mask_bits: np.ndarray    # [N, ceil(N/64)] uint64: bit j%64 of word j//64 of row i


def select_top(state: DraftState, m: int) -> np.ndarray:
    """Ids of the m candidates of highest value, ties to the lower id (= shallower)."""
    ids = np.arange(state.score.shape[0])
    return np.lexsort((ids, -state.score))[:m]


def select_frontiers(state: DraftState, rank_by_value: bool = True) -> np.ndarray:
    """The "w/o reranking" ablation of Section 5.2: the draft is what the expansion
    phase itself selected -- every layer's k best nodes (the frontiers, plus the k
    best of the last layer, which is never expanded).  The last layer is ranked the
    way the expansion phase ranks: by value, or by the nodes' own confidence when
    value is switched off too ("w/o both" in Table 3)."""
    k, D = state.topk, state.depth
    ids = [int(c) for c in state.frontier[1:].reshape(-1) if c >= 0]
    last = np.arange(cand_base(D - 1, k), n_candidates(D, k))
    key = state.score[last] if rank_by_value else state.own[last]
    ids += [int(c) for c in last[np.lexsort((last, -key))[:k]]]
    return np.array(sorted(set(ids)), dtype=np.int64)


def flatten(state: DraftState, selected: np.ndarray, root_token: int, prefix_len: int) -> FlatTree:
    """Lay the root and the selected candidates out as a 1-D sequence (increasing
    candidate id, so parents precede children) and build the mask under which each
    row sees exactly itself and its ancestors."""
    k = state.topk
    sel = np.sort(np.asarray(selected, dtype=np.int64))
    n = sel.shape[0] + 1
    row_of = {int(c): i + 1 for i, c in enumerate(sel)}
    token = np.empty(n, dtype=np.int64)
    parent = np.empty(n, dtype=np.int64)
    depth = np.empty(n, dtype=np.int64)
    cand = np.empty(n, dtype=np.int64)
    token[0], parent[0], depth[0], cand[0] = root_token, -1, 0, -1
    for i, c in enumerate(sel, start=1):
        c = int(c)
        token[i] = state.token[c]
        cand[i] = c
        depth[i] = cand_depth(c, k)
        p = int(state.parent[c])
        parent[i] = 0 if p < 0 else row_of[p]       # KeyError here = selection not ancestor-closed
    mask = np.zeros((n, n), dtype=bool)
    for i in range(n):
        j = i
        while j >= 0:                                # walk to the root
            mask[i, j] = True
            j = int(parent[j])
    words = (n + 63) // 64
    bits = np.zeros((n, words), dtype=np.uint64)
    for i in range(n):
        for j in range(n):
            if mask[i, j]:
                bits[i, j // 64] |= np.uint64(1) << np.uint64(j % 64)
    return FlatTree(token, parent, depth, cand, prefix_len + depth, mask, bits)


def static_shape(nodes, depth: int, topk: int):
    """A fixed tree shape given as a list of (parent position in the list or -1, rank among the
    parent's children), parents before children, as candidate ids: returns (ids of the nodes in
    list order, frontier [depth, topk] with the expanded nodes of every layer in order of first
    use, -1 padded)."""
    ids: List[int] = []
    node_depth: List[int] = []
    frontier = np.full((depth, topk), -1, dtype=np.int64)
    used = [0] * (depth + 1)
    slot_of = {}
    for par, rank in nodes:
        assert 0 <= rank < topk and par < len(ids)
        if par < 0:
            ids.append(rank)
            node_depth.append(1)
            continue
        d = node_depth[par]                                   # the parent's depth = the pass that expands it
        assert d < depth, "a node of the deepest layer cannot have children"
        if par not in slot_of:
            assert used[d] < topk, "more than k expanded nodes in one layer"
            slot_of[par] = used[d]
            frontier[d, used[d]] = ids[par]
            used[d] += 1
        ids.append(cand_base(d, topk) + slot_of[par] * topk + rank)
        node_depth.append(d + 1)
    return np.array(ids, dtype=np.int64), frontier


def rerank(state: DraftState, n_tree: int, root_token: int, prefix_len: int,
           use_rerank: bool = True, rank_by_value: bool = True, static_sel=None) -> FlatTree:
    """Top-(n_tree - 1) of all candidates by value, flattened behind the root.
    use_rerank=False: the expansion phase's own selection (n_tree is then D*k + 1).
    static_sel: the nodes of a fixed shape (Section 2.2), no selection at all."""
    if static_sel is not None:
        return flatten(state, np.asarray(static_sel, dtype=np.int64), root_token, prefix_len)
    sel = select_top(state, n_tree - 1) if use_rerank else select_frontiers(state, rank_by_value)
    return flatten(state, sel, root_token, prefix_len)


# ----------------------------------------------------------------------------
# tree attention (Section 4.2: ancestor-only visibility)
# ----------------------------------------------------------------------------

def tree_attn(Q, K_prefix, V_prefix, K_tree, V_tree, mask, scale: Optional[float] = None):
    """Attention of the N tree rows over the P prefix keys (all visible) and the N
    tree keys (visible where mask[i, j]).

    Q [N, Hq, dh]; K/V_prefix [P, Hkv, dh]; K/V_tree [N, Hkv, dh]; mask [N, N] bool.
    Query head h reads KV head h // (Hq // Hkv).  Returns O [N, Hq, dh] and the
    log-sum-exp of the scaled scores, lse [N, Hq].  Two-pass softmax in float64.
    """
    Q = np.asarray(Q, dtype=np.float64)
    Kp = np.asarray(K_prefix, dtype=np.float64)
    Vp = np.asarray(V_prefix, dtype=np.float64)
    Kt = np.asarray(K_tree, dtype=np.float64)
    Vt = np.asarray(V_tree, dtype=np.float64)
    mask = np.asarray(mask, dtype=bool)
    N, Hq, dh = Q.shape
    Hkv = Kt.shape[1]
    group = Hq // Hkv
    if scale is None or scale == 0:
        scale = 1.0 / np.sqrt(dh)
    O = np.empty((N, Hq, dh), dtype=np.float64)
    lse = np.empty((N, Hq), dtype=np.float64)
    for h in range(Hq):
        g = h // group
        s_pre = (Q[:, h, :] @ Kp[:, g, :].T) * scale            # [N, P]
        s_tree = (Q[:, h, :] @ Kt[:, g, :].T) * scale           # [N, N]
        s_tree = np.where(mask, s_tree, -np.inf)
        s = np.concatenate([s_pre, s_tree], axis=1)
        vals = np.concatenate([Vp[:, g, :], Vt[:, g, :]], axis=0)
        m = np.max(s, axis=1, keepdims=True)
        w = np.exp(s - m)
        z = np.sum(w, axis=1, keepdims=True)
        O[:, h, :] = (w @ vals) / z
        lse[:, h] = (m + np.log(z))[:, 0]
    return O, lse


# ----------------------------------------------------------------------------
# acceptance (Sections 2.1 and 2.2)
# ----------------------------------------------------------------------------

@dataclass
class AcceptResult:
    accept_len: int                # number of accepted draft tokens
    path: List[int]                # flat rows from the root to the last accepted node
    bonus_token: int               # the token emitted after the accepted path
    trace: Optional[list] = None   # sampling only: per tested child (row, accept probability)
    final_p: Optional[np.ndarray] = None   # sampling only: distribution the bonus was drawn from
    ratios: Optional[dict] = None  # sampling only: tested row -> p(x)/q(x) before the cap at 1 (for reports)


def _children(tree_parent: np.ndarray, cur: int) -> List[int]:
    return [int(c) for c in np.nonzero(np.asarray(tree_parent) == cur)[0]]


def accept_greedy(target_logits, tree_token, tree_parent) -> AcceptResult:
    """Temperature 0: the target's choice after a row is the arg-max of its logits
    (lowest id on ties).  From the root, step to the child carrying that token
    while there is one; the token chosen at the last accepted row is emitted."""
    tl = np.asarray(target_logits, dtype=np.float64)
    tree_token = np.asarray(tree_token)
    choice = np.argmax(tl, axis=1)                     # first maximum = lowest id
    cur, path = 0, [0]
    while True:
        nxt = [c for c in _children(tree_parent, cur) if int(tree_token[c]) == int(choice[cur])]
        if not nxt:
            break
        cur = nxt[0]
        path.append(cur)
    return AcceptResult(len(path) - 1, path, int(choice[cur]))


def accept_sample(target_logits, draft_logits, temperature: float, u_accept, u_bonus,
                  tree_token, tree_parent, tree_cand, topk: int) -> AcceptResult:
    """Sampling regime: speculative sampling applied along the tree.

    At the current row, p is the target distribution softmax(logits / T) and q the
    draft distribution its children were taken from (softmax of the draft logits
    at temperature 1).  Children are tried in flat order.  A child with token x is
    accepted with probability min(1, p(x) / q(x)) (Section 2.1) -- decided as
    u_accept[child] < p(x)/q(x).  After a rejection the target is replaced by the
    residual norm(max(0, p - q)) (Section 2.1), the rejected token is removed from
    q and q renormalised (siblings are distinct tokens, i.e. drawn without
    replacement), and the next sibling is tried (Section 2.2).  When no child is
    left the emitted token is drawn from the current p by inverse CDF with
    u_bonus[current row].
    """
    tl = np.asarray(target_logits, dtype=np.float64)
    dl = np.asarray(draft_logits, dtype=np.float64)
    tree_token = np.asarray(tree_token)
    tree_cand = np.asarray(tree_cand)
    T = float(temperature)
    cur, path, trace, ratios = 0, [0], [], {}
    while True:
        p = softmax64(tl[cur] / T)
        kids = _children(tree_parent, cur)
        moved = False
        if kids:
            q = softmax64(dl[parent_draft_row(int(tree_cand[kids[0]]), topk)])
            for c in kids:
                x = int(tree_token[c])
                ratio = p[x] / q[x]
                trace.append((c, min(1.0, ratio)))
                ratios[c] = float(ratio)
                if float(u_accept[c]) < ratio:
                    cur = c
                    path.append(c)
                    moved = True
                    break
                resid = np.maximum(p - q, 0.0)
                tot = resid.sum()
                if tot > 0.0:
                    p = resid / tot
                q = q.copy()
                q[x] = 0.0
                qs = q.sum()
                if qs > 0.0:
                    q = q / qs
        if not moved:
            total = p.sum()
            cdf = np.cumsum(p)
            hit = np.nonzero(cdf > float(u_bonus[cur]) * total)[0]
            bonus = int(hit[0]) if hit.size else int(np.nonzero(p > 0.0)[0][-1])
            return AcceptResult(len(path) - 1, path, bonus, trace, p, ratios)


# ----------------------------------------------------------------------------
# what a round leaves behind (Section 2.1: keep the accepted tokens, discard the rest)
# ----------------------------------------------------------------------------

def commit_kv(K_cache, V_cache, region_start: int, region_end: int, prefix_len: int,
              K_tree, V_tree, path) -> int:
    """Appends the keys/values of the accepted rows to the sequence's region of a
    pre-allocated cache.  `path` is the accepted path in flat rows, root first: the
    root is the last committed token, whose key/value this verification pass
    computed, so len(path) = accept_len + 1 rows are appended behind the prefix_len
    rows already there.  Rows of rejected branches are not copied anywhere.  Rows
    that would fall outside the region are dropped.  Returns the new prefix length
    (of the rows that fitted)."""
    n = int(prefix_len)
    for row in path:
        dst = region_start + n
        if dst >= region_end:
            break
        K_cache[dst] = K_tree[int(row)]
        V_cache[dst] = V_tree[int(row)]
        n += 1
    return n


@dataclass
class RoundOutput:
    tokens: List[int]        # tokens this round adds to the text: the accepted draft tokens, then the bonus token
    root_token: int          # root of the next round's tree = the bonus token
    prefix_len: int          # KV rows after the round
    next_hidden: Optional[np.ndarray]   # target feature at the last accepted row (input of the next draft)


def commit_round(tree_token, path, bonus_token: int, prefix_len: int, target_hidden=None) -> RoundOutput:
    """The accepted draft tokens are kept, followed by the token the target emitted
    at the last accepted row (Section 2.1); it becomes the next root.  The KV prefix
    grows by the root and the accepted tokens (the bonus token has no key yet)."""
    toks = [int(tree_token[int(r)]) for r in path[1:]] + [int(bonus_token)]
    nh = None if target_hidden is None else np.array(target_hidden[int(path[-1])], copy=True)
    return RoundOutput(toks, int(bonus_token), int(prefix_len) + len(path), nh)
