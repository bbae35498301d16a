"""Lock-step comparison of the HIP path with the CPU oracle (used by the GPU tests,
the smoke check and the benchmark's self-check).

Structure (token ids, parents, mask, accepted path) must be bit-exact except for
swaps between candidates whose ORACLE scores differ by less than SWAP_TOL = 1e-5.
To make that checkable, the comparison runs in lock-step: after every GPU expand
pass the GPU's choices are checked for admissibility under the oracle's float64
log-probabilities, and the oracle's state is then continued from the GPU's choice
(its own float64 scores for the GPU's tokens), so one admissible swap cannot
cascade into later mismatches.  Floating-point outputs are compared with
max |gpu - ref| / max(|ref|, rms(ref)) <= 1e-4 (fp32 inputs) or 2e-2 (bf16 inputs).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List

import numpy as np
import torch

from oracle import eagle2_oracle as orc

SWAP_TOL = 1e-5
REL_TOL = {"fp32": 1e-4, "bf16": 2e-2}
# Raw logits and joint scores are float32 sums of exactly representable products (bf16 x bf16, or
# float32 inputs) plus float64 adds: their error does not depend on the I/O type, so both are held
# to the float32 bound (measured: logits 2e-6, scores 4e-7 relative).
LOGIT_TOL = 1e-4
SCORE_TOL = 1e-4
DECISION_TOL = 1e-5     # a sampling decision may differ only if |u - p/q| < DECISION_TOL * max(1, p/q)


def f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a tensor's stored values to float64 on the host."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    ref = np.asarray(ref, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    den = np.maximum(np.abs(ref), max(rms, 1e-300))
    return float(np.max(np.abs(got - ref) / den))


@dataclass
class Report:
    swaps_topk: int = 0          # per-row top-k positions where the GPU token differs from the oracle's
    swaps_frontier: int = 0
    swaps_rerank: int = 0
    max_score_err: float = 0.0   # absolute, joint scores
    max_logit_rel: float = 0.0
    max_attn_rel: float = 0.0
    max_lse_err: float = 0.0
    near_threshold_decisions: int = 0    # sampling decisions that differ from the oracle's within DECISION_TOL
    notes: List[str] = field(default_factory=list)
    # the oracle's own float64 draft logits per sequence ([R, V]), filled pass by pass
    oracle_draft_logits: dict = field(default_factory=dict)


def _admissible(picked_vals: np.ndarray, all_vals: np.ndarray, picked_idx: np.ndarray, what: str):
    """picked_* in the GPU's rank order; values are the oracle's.  The pick is admissible
    if it is sorted up to SWAP_TOL and nothing left out beats the worst pick by SWAP_TOL."""
    assert len(set(picked_idx.tolist())) == len(picked_idx), f"{what}: duplicate picks {picked_idx}"
    d = np.diff(picked_vals)
    assert np.all(d <= SWAP_TOL), f"{what}: GPU order violates oracle values by {d.max():.3e}"
    rest = np.delete(all_vals, picked_idx)
    if rest.size:
        assert rest.max() <= picked_vals.min() + SWAP_TOL, \
            f"{what}: a candidate left out beats a pick by {rest.max() - picked_vals.min():.3e}"


FLAG_RANK_BY_CONFIDENCE, FLAG_NO_RERANK = 1, 2      # the C ABI's ablation switches (Section 5.2)
FLAG_STATIC_TREE = 4                                # fixed-shape tree (Section 2.2)


def check_expand_pass(rnd, cfg, states, d: int, H64_d: np.ndarray, W64: np.ndarray, report: Report,
                      check_logits: bool = True, flags: int = 0, static_frontier=None):
    """Checks the GPU's expand pass d (already run; H64_d [B, F, Hd] are the hidden states it was
    given, widened to float64) against the oracle, and continues the oracle states from the GPU's
    choices."""
    B, D, k = cfg.batch, cfg.depth, cfg.topk
    by_value = not (flags & FLAG_RANK_BY_CONFIDENCE)
    g_tok = rnd.cand_token.cpu().numpy()
    g_score = rnd.cand_score.cpu().numpy()
    g_par = rnd.cand_parent.cpu().numpy()
    g_front = rnd.frontier.cpu().numpy()
    F = 1 if d == 0 else k
    base = orc.cand_base(d, k)
    for b in range(B):
        st = states[b]
        ref = st.copy()
        keep = check_logits and rnd.draft_logits is not None
        dl_ref = report.oracle_draft_logits.setdefault(b, np.zeros((orc.n_draft_rows(D, k), cfg.vocab))) if keep else None
        sf = None if static_frontier is None or d + 1 >= D else static_frontier[d + 1]
        logp = orc.expand(ref, d, H64_d[b, :F], W64, draft_logits=dl_ref, rank_by_value=by_value, static_frontier=sf)
        if dl_ref is not None:
            # the dense draft logits are the draft distribution of the acceptance rule (Section 2.1):
            # every row this pass owns must hold the oracle's logits of that (sequence, slot)
            rows = [orc.draft_row(d, s, k) for s in range(F)]
            got = rnd.draft_logits[b, rows].cpu().numpy().astype(np.float64)
            assert np.all(np.isfinite(got)), f"seq {b} pass {d}: draft-logit rows left unwritten or not finite"
            for i, r in enumerate(rows):
                e = rel_err(got[i], dl_ref[r])
                report.max_logit_rel = max(report.max_logit_rel, e)
                assert e <= LOGIT_TOL, f"seq {b} pass {d} slot {i}: draft logits (row {r}) rel err {e:.3e} > {LOGIT_TOL}"
        for s in range(F):
            if d > 0 and int(st.frontier[d, s]) < 0:
                continue                                    # unused slot of a fixed shape: its candidates are never read
            ids = base + s * k + np.arange(k)
            picks = g_tok[b, ids].astype(np.int64)
            assert picks.min() >= 0 and picks.max() < cfg.vocab, f"pass {d} row {s}: token out of range"
            _admissible(logp[s, picks], logp[s], picks, f"seq {b} pass {d} row {s} top-k")
            report.swaps_topk += int(np.sum(picks != ref.token[ids]))
            par = -1 if d == 0 else int(st.frontier[d, s])
            assert np.all(g_par[b, ids] == par), f"seq {b} pass {d} row {s}: parent ids differ"
            par_score = 0.0 if d == 0 else float(st.score[par])
            st.token[ids] = picks
            st.parent[ids] = par
            st.score[ids] = par_score + logp[s, picks]          # oracle values for the GPU's picks
            st.own[ids] = logp[s, picks]
            err = np.abs(g_score[b, ids] - st.score[ids])
            report.max_score_err = max(report.max_score_err, float(err.max()))
            assert np.all(err <= SCORE_TOL * np.maximum(np.abs(st.score[ids]), 1.0)), \
                f"seq {b} pass {d} row {s}: joint score error {err.max():.3e}"
        if d + 1 < D and static_frontier is not None:
            assert np.array_equal(g_front[b, d + 1], static_frontier[d + 1]), f"seq {b} pass {d}: the fixed frontier was overwritten"
            st.frontier[d + 1] = static_frontier[d + 1]
        elif d + 1 < D:
            new = base + np.arange(F * k)
            gf = g_front[b, d + 1].astype(np.int64)
            assert gf.min() >= base and gf.max() < base + F * k, f"seq {b} pass {d}: frontier outside the new layer"
            key = st.score if by_value else st.own
            _admissible(key[gf], key[new], gf - base, f"seq {b} pass {d} frontier")
            want = new[np.lexsort((new, -key[new]))[:k]]
            report.swaps_frontier += int(np.sum(gf != want))
            st.frontier[d + 1] = gf


def lockstep_expand(rnd, cfg, H_all: torch.Tensor, W: torch.Tensor, W64: np.ndarray = None,
                    report: Report = None, check_logits: bool = True, flags: int = 0, static_frontier=None):
    """Runs the D expand passes on the GPU, checking each against the oracle.
    Returns (oracle states continued from the GPU's choices, report)."""
    report = report or Report()
    B, D, k = cfg.batch, cfg.depth, cfg.topk
    if W64 is None:
        W64 = f64(W)
    H64 = f64(H_all)
    states = [orc.DraftState(D, k) for _ in range(B)]
    dl = rnd.draft_logits if check_logits else None
    report.oracle_draft_logits.clear()
    if dl is not None:
        dl.fill_(float("nan"))                          # a row no pass writes stays NaN and fails the checks
    for d in range(D):
        before = dl.clone() if dl is not None else None
        rnd.expand(d, H_all[:, d], W, h_seq_stride=D * k * cfg.hidden)
        if H_all.is_cuda:
            torch.cuda.synchronize()
        if dl is not None:
            # pass d owns rows draft_row(d, 0..F-1) and must leave every other row bit for bit as it was
            own = [orc.draft_row(d, s, k) for s in range(1 if d == 0 else k)]
            other = [r for r in range(dl.shape[1]) if r not in own]
            same = torch.equal(dl[:, other].view(torch.int32), before[:, other].view(torch.int32))
            assert same, f"pass {d} changed draft-logit rows that belong to other passes"
        check_expand_pass(rnd, cfg, states, d, H64[:, d], W64, report, check_logits, flags, static_frontier)
    return states, report


def check_rerank(rnd, cfg, states, root_token: np.ndarray, prefix_len: np.ndarray, report: Report, flags: int = 0,
                 static_sel=None):
    """GPU rerank vs oracle: admissible selection, then bit-exact flattening of that selection."""
    B, N, k = cfg.batch, cfg.n_tree, cfg.topk
    t_tok = rnd.tree_token.cpu().numpy()
    t_par = rnd.tree_parent.cpu().numpy()
    t_dep = rnd.tree_depth.cpu().numpy()
    t_cand = rnd.tree_cand.cpu().numpy()
    t_pos = rnd.position_ids.cpu().numpy()
    t_mask = rnd.mask_bits.cpu().numpy().view(np.uint64)
    trees = []
    for b in range(B):
        st = states[b]
        sel = t_cand[b, 1:].astype(np.int64)
        assert t_cand[b, 0] == -1 and sel.min() >= 0 and sel.max() < cfg.n_cand
        assert np.all(np.diff(sel) > 0), "flat order must be increasing candidate id"
        if static_sel is not None:
            assert np.array_equal(sel, np.sort(static_sel)), f"seq {b}: tree nodes differ from the fixed shape"
            want = np.sort(static_sel)
        elif flags & FLAG_NO_RERANK:
            # the expansion phase's own selection: every frontier, plus an admissible top-k of the last layer
            D = cfg.depth
            assert N == D * k + 1
            lbase = orc.cand_base(D - 1, k)              # first id of the last layer
            picked = sel[sel >= lbase]
            assert set(sel[sel < lbase].tolist()) == set(st.frontier[1:].reshape(-1).tolist()), \
                f"seq {b}: rows of layers 1..D-1 are not the expanded frontiers"
            assert len(picked) == k, f"seq {b}: {len(picked)} last-layer nodes selected, expected {k}"
            key = st.score if not (flags & FLAG_RANK_BY_CONFIDENCE) else st.own
            order = np.lexsort((picked, -key[picked]))
            _admissible(key[picked][order], key[lbase:], picked[order] - lbase, f"seq {b} last-layer top-k")
            want = orc.select_frontiers(st, not (flags & FLAG_RANK_BY_CONFIDENCE))
        else:
            order = np.lexsort((sel, -st.score[sel]))
            _admissible(st.score[sel][order], st.score, sel[order], f"seq {b} rerank")
            want = np.sort(orc.select_top(st, N - 1))
        report.swaps_rerank += int(np.sum(sel != want))
        tree = orc.flatten(st, sel, int(root_token[b]), int(prefix_len[b]))
        assert np.array_equal(t_tok[b], tree.token), f"seq {b}: tree tokens differ"
        assert np.array_equal(t_par[b], tree.parent), f"seq {b}: tree parents differ"
        assert np.array_equal(t_dep[b], tree.depth), f"seq {b}: tree depths differ"
        assert np.array_equal(t_pos[b], tree.position), f"seq {b}: position ids differ"
        assert np.array_equal(t_mask[b], tree.mask_bits), f"seq {b}: ancestor mask differs"
        trees.append(tree)
    return trees


def check_attention(cfg, trees, Q, Kp, Vp, Kt, Vt, kv_offsets, O, lse, report: Report,
                    seqs=None, heads=None, prefix_lens=None):
    """GPU attention output vs oracle, for all or a sample of (sequence, head).
    prefix_lens: filled rows per region when the KV buffer is a pre-allocated cache."""
    off = kv_offsets.cpu().numpy()
    tol = REL_TOL[cfg.dtype]
    g = cfg.n_q_heads // cfg.n_kv_heads
    for b in (range(cfg.batch) if seqs is None else seqs):
        lo, hi = int(off[b]), int(off[b + 1])
        if prefix_lens is not None:
            hi = lo + int(prefix_lens[b])
        hq = list(range(cfg.n_q_heads)) if heads is None else list(heads)
        kvh = sorted({h // g for h in hq})
        # the oracle maps head h -> kv head h // g; feed it the needed kv heads with g preserved
        remap = {kh: i for i, kh in enumerate(kvh)}
        q_sel = []
        for kh in kvh:
            q_sel += list(range(kh * g, (kh + 1) * g))
        Oq, lq = orc.tree_attn(f64(Q[b][:, q_sel]), f64(Kp[lo:hi][:, kvh]), f64(Vp[lo:hi][:, kvh]),
                               f64(Kt[b][:, kvh]), f64(Vt[b][:, kvh]), trees[b].mask)
        for h in hq:
            col = remap[h // g] * g + (h % g)
            e = rel_err(f64(O[b, :, h]), Oq[:, col])
            report.max_attn_rel = max(report.max_attn_rel, e)
            assert e <= tol, f"seq {b} head {h}: attention rel err {e:.3e} > {tol}"
            if lse is not None:
                le = float(np.max(np.abs(f64(lse[b, :, h]) - lq[:, col])))
                report.max_lse_err = max(report.max_lse_err, le)
                assert le <= tol * max(1.0, float(np.max(np.abs(lq[:, col])))), f"seq {b} head {h}: lse err {le:.3e}"


def _trim(path) -> list:
    return [int(r) for r in path if int(r) >= 0]


def _check_bonus(b, got: int, res, u: float, report: Report, what: str):
    """The emitted token must be the oracle's, or sit across a CDF edge that the draw touches
    within DECISION_TOL of the total mass."""
    if got == res.bonus_token:
        return
    assert res.final_p is not None, f"seq {b}: bonus {got} != {res.bonus_token} ({what})"
    p = res.final_p
    cdf = np.cumsum(p) / p.sum()
    lo, hi = min(got, res.bonus_token), max(got, res.bonus_token)
    assert 0 <= lo and hi < len(p), f"seq {b}: bonus {got} out of range ({what})"
    assert abs(cdf[lo] - u) < DECISION_TOL and np.all(p[lo + 1:hi] <= DECISION_TOL), \
        f"seq {b}: bonus {got} != {res.bonus_token} and not at a CDF edge ({what})"
    report.notes.append(f"seq {b}: bonus differs at a CDF edge ({what})")


def check_accept(rnd, cfg, trees, modes, target_logits, temperature, u_accept, u_bonus, report: Report):
    """Greedy: bit-exact.  Sampling is checked twice.  (1) Fed the float32 draft logits the GPU
    itself produced, the oracle must reproduce path, length and emitted token.  (2) Fed its OWN
    float64 draft logits (kept by check_expand_pass), the oracle must take the same decisions,
    except at a child whose uniform lies within DECISION_TOL * max(1, p/q) of the ratio p/q, or a
    bonus draw within DECISION_TOL of a CDF edge; such cases are counted, and what follows the
    first of them cannot be compared (the two walks are then in different subtrees)."""
    B, D, k = cfg.batch, cfg.depth, cfg.topk
    a_len = rnd.accept_len.cpu().numpy()
    a_path = rnd.accept_path.cpu().numpy()
    a_bonus = rnd.bonus_token.cpu().numpy()
    out = []
    for b in range(B):
        tree = trees[b]
        tl = f64(target_logits[b])
        if modes[b] == 0:
            res = orc.accept_greedy(tl, tree.token, tree.parent)
        else:
            res = orc.accept_sample(tl, f64(rnd.draft_logits[b]), float(temperature[b]), f64(u_accept[b]),
                                    f64(u_bonus[b]), tree.token, tree.parent, tree.cand, k)
        want_path = res.path + [-1] * (D + 1 - len(res.path))
        assert a_len[b] == res.accept_len, f"seq {b}: accept_len {a_len[b]} != {res.accept_len}"
        assert a_path[b].tolist() == want_path, f"seq {b}: path {a_path[b].tolist()} != {want_path}"
        if modes[b] == 1:
            _check_bonus(b, int(a_bonus[b]), res, float(u_bonus[b][res.path[-1]]), report, "oracle on the GPU's draft logits")
        else:
            assert a_bonus[b] == res.bonus_token, f"seq {b}: bonus {a_bonus[b]} != {res.bonus_token}"
        if modes[b] == 1 and b in report.oracle_draft_logits:
            own = orc.accept_sample(tl, report.oracle_draft_logits[b], float(temperature[b]), f64(u_accept[b]),
                                    f64(u_bonus[b]), tree.token, tree.parent, tree.cand, k)
            got = _trim(a_path[b])
            if got == own.path:
                _check_bonus(b, int(a_bonus[b]), own, float(u_bonus[b][own.path[-1]]), report, "oracle on its own draft logits")
            else:
                i = 0
                while i < min(len(got), len(own.path)) and got[i] == own.path[i]:
                    i += 1
                assert i >= 1, f"seq {b}: the accepted path does not start at the root"
                cur = own.path[i - 1]
                kids = [int(c) for c in np.nonzero(np.asarray(tree.parent) == cur)[0]]
                taken = [kids.index(x[i]) for x in (got, own.path) if i < len(x) and x[i] in kids]
                assert taken, f"seq {b}: paths {got} / {own.path} part at row {cur} without a child of it"
                c = kids[min(taken)]                    # the first sibling on which the two decisions differ
                ratio, u = own.ratios[c], float(u_accept[b][c])
                assert abs(u - ratio) < DECISION_TOL * max(1.0, ratio), \
                    f"seq {b}: path {got} != oracle's {own.path} on its own draft logits; decision at row {c}: " \
                    f"u = {u:.9f}, p/q = {ratio:.9f}"
                report.near_threshold_decisions += 1
                report.notes.append(f"seq {b}: decision at row {c} within tolerance of its threshold")
        out.append(res)
    return out


# ---------------------------------------------------------------------------------------
# a whole round: GPU calls in the method's order, each stage checked against the oracle
# ---------------------------------------------------------------------------------------

def run_and_check_round(cfg, device="cuda", h_scale: float = 1.0, plant: bool = False,
                        layers=(0,), attn_seqs=None, attn_heads=None, W=None, W64=None, verbose=True,
                        round_factory=None, flags: int = 0, static_nodes=None):
    """Runs one draft-plus-verify round of `cfg` on the GPU and checks every stage.
    plant=True plants the target's preferred tokens along a tree path so that sequence b
    accepts min(b mod (D+1), deepest available) tokens in greedy mode."""
    import workloads as wl
    if round_factory is None:
        from paper_2406_16858_amd import DraftRound as round_factory

    def sync():
        if torch.device(device).type == "cuda":
            torch.cuda.synchronize()

    rep = Report()
    B, D, k, N, V = cfg.batch, cfg.depth, cfg.topk, cfg.n_tree, cfg.vocab
    if W is None:
        W = wl.make_lm_head(cfg, device)
    H_all = wl.make_hidden_states(cfg, device, scale=h_scale)
    plens = wl.make_prefix_lengths(cfg)
    modes_l = {"greedy": [0] * B, "sample": [1] * B, "mixed": [b % 2 for b in range(B)]}[cfg.accept]
    extra = {"flags": flags} if flags else {}
    static_sel = static_front = None
    if static_nodes is not None:
        # a fixed shape (list of (parent position, rank)): the caller owns the frontiers and the node list
        static_sel, static_front = orc.static_shape(static_nodes, D, k)
        assert len(static_sel) == N - 1
        extra["static_tree"] = torch.from_numpy(np.sort(static_sel).astype(np.int32)).to(device)
    rnd = round_factory(B, V, cfg.hidden, D, k, N, cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     total_prefix=sum(plens), keep_draft_logits=any(modes_l), device=device, **extra)
    if static_front is not None:
        rnd.frontier.copy_(torch.from_numpy(np.tile(static_front.astype(np.int32), (B, 1, 1))))
    states, rep = lockstep_expand(rnd, cfg, H_all, W, W64=W64, report=rep, flags=flags, static_frontier=static_front)

    root = torch.arange(B, dtype=torch.int32) * 3 + 7
    plen_t = torch.tensor(plens, dtype=torch.int32)
    rnd.rerank(root.to(device), plen_t.to(device))
    sync()
    trees = check_rerank(rnd, cfg, states, root.numpy(), plen_t.numpy(), rep, flags=flags, static_sel=static_sel)

    for layer in layers:
        Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, device, layer=layer, prefix_lens=plens)
        O = torch.full_like(Q, float("nan"))
        lse = torch.full((B, N, cfg.n_q_heads), float("nan"), dtype=torch.float32, device=device)
        rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse)
        sync()
        assert not torch.isnan(O.float()).any(), "attention left outputs unwritten"
        check_attention(cfg, trees, Q, Kp, Vp, Kt, Vt, off, O, lse, rep, seqs=attn_seqs, heads=attn_heads)
        del Q, Kp, Vp, Kt, Vt, O

    tl, _ = wl.make_target_logits(cfg, device)
    if plant:
        for b in range(B):
            tree = trees[b]
            deepest = int(np.argmax(tree.depth))
            chain = []
            j = deepest
            while j >= 0:
                chain.append(j)
                j = int(tree.parent[j])
            chain.reverse()
            L = min(b % (D + 1) if B > 1 else len(chain) - 1, len(chain) - 1)
            for i in range(L):
                row = tl[b, chain[i]]
                row[int(tree.token[chain[i + 1]])] = row.max() + 8.0
    ua, ub = wl.make_uniforms(cfg, device)
    temp = torch.full((B,), cfg.temperature, dtype=torch.float32, device=device)
    mode_t = torch.tensor(modes_l, dtype=torch.int32, device=device)
    rnd.accept(mode_t, tl, temp, ua, ub)
    sync()
    results = check_accept(rnd, cfg, trees, modes_l, tl, temp.cpu().numpy(), ua, ub, rep)
    if verbose:
        lens = [r.accept_len for r in results]
        print(f"[{cfg.name} scale={h_scale} plant={plant}] swaps topk/frontier/rerank = "
              f"{rep.swaps_topk}/{rep.swaps_frontier}/{rep.swaps_rerank}  score_err={rep.max_score_err:.2e} "
              f"logit_rel={rep.max_logit_rel:.2e} attn_rel={rep.max_attn_rel:.2e} lse_err={rep.max_lse_err:.2e} "
              f"near_thr={rep.near_threshold_decisions} accept_len={lens} depth_hist={np.bincount(trees[0].depth).tolist()} {rep.notes}", flush=True)
    return rep, trees, results
