"""GPU edge cases through the C ABI: determinism, the largest supported shapes, error
returns that must not enqueue anything, and sequences that accept with both modes."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl
from tests.parity_utils import run_and_check_round

pytestmark = pytest.mark.gpu


def _cfg(name, **kw):
    base = dict(name=name, index=0, dtype="bf16", batch=1, vocab=4096, hidden=512, depth=4, topk=5, n_tree=24,
                n_q_heads=8, n_kv_heads=2, head_dim=64, prefix_lo=130, prefix_hi=130, n_layers=1, w_std=0.05,
                accept="greedy", temperature=1.0, seed=4321)
    base.update(kw)
    return wl.RoundConfig(**base)


def test_largest_candidate_count_and_tree():
    # C = 16 + 7*256 = 1808 candidates, N = 128 rows (two mask words), 33 rejections possible at most
    cfg = _cfg("max_cand", topk=16, depth=8, n_tree=128, vocab=3000, accept="sample", seed=12)
    run_and_check_round(cfg, h_scale=6.0)


def test_smallest_shapes():
    cfg = _cfg("min_shapes", vocab=16, topk=1, depth=1, n_tree=2, hidden=512, n_q_heads=1, n_kv_heads=1,
               prefix_lo=0, prefix_hi=0, seed=2)
    run_and_check_round(cfg, h_scale=2.0)
    cfg = _cfg("vocab_eq_topk", vocab=16, topk=16, depth=2, n_tree=20, accept="sample", seed=3)
    run_and_check_round(cfg, h_scale=2.0)


def test_many_sequences_ragged_and_long_prefix():
    cfg = _cfg("batch9", batch=9, accept="mixed", prefix_lo=0, prefix_hi=9000, n_q_heads=8, n_kv_heads=8,
               head_dim=128, n_tree=30, seed=21)
    run_and_check_round(cfg, h_scale=6.0, plant=True)


def test_many_small_sequences():
    # 257 sequences: more sequences than compute units, 514 frontier rows (four passes of the many-row LM head
    # per expansion), one sampling workgroup per sequence
    cfg = _cfg("batch257", batch=257, vocab=300, hidden=512, depth=2, topk=2, n_tree=5, n_q_heads=2, n_kv_heads=1,
               head_dim=64, prefix_lo=0, prefix_hi=40, accept="mixed", seed=31)
    run_and_check_round(cfg, h_scale=4.0, verbose=False)


def test_sampling_with_more_vocabulary_per_thread_than_registers_hold():
    # 40 sampling sequences share the chip: 12 workgroups each, 50021 / 12 / 256 > 16 entries per thread, so the
    # sampling kernel rebuilds its state from the logits in every pass instead of keeping it in registers
    cfg = _cfg("uncached_sampling", batch=40, vocab=50021, hidden=512, depth=2, topk=3, n_tree=8, n_q_heads=2, n_kv_heads=1,
               head_dim=64, prefix_lo=0, prefix_hi=30, accept="sample", temperature=0.8, seed=41)
    run_and_check_round(cfg, h_scale=5.0, verbose=False)


def test_bitwise_determinism():
    from paper_2406_16858_amd import DraftRound
    cfg = wl.get_config(2)
    W = wl.make_lm_head(cfg, "cuda")
    H = wl.make_hidden_states(cfg, "cuda", scale=6.0)
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda")
    tl, _ = wl.make_target_logits(cfg, "cuda")
    ua, ub = wl.make_uniforms(cfg, "cuda")
    outs = []
    for rep in range(3):
        rnd = DraftRound(1, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, cfg.n_tree, cfg.dtype, cfg.n_q_heads,
                         cfg.n_kv_heads, cfg.head_dim, total_prefix=cfg.prefix_lo, keep_draft_logits=True)
        rnd.workspace.fill_(rep * 37 + 1)                  # the workspace carries nothing between calls
        rnd.expand_all(H, W)
        rnd.rerank(torch.tensor([5], dtype=torch.int32, device="cuda"),
                   torch.tensor([cfg.prefix_lo], dtype=torch.int32, device="cuda"))
        O = torch.empty_like(Q)
        lse = torch.empty((1, cfg.n_tree, cfg.n_q_heads), dtype=torch.float32, device="cuda")
        rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse)
        mode = torch.ones(1, dtype=torch.int32, device="cuda")
        rnd.accept(mode, tl, torch.ones(1, device="cuda"), ua, ub)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (rnd.cand_token, rnd.cand_score, rnd.frontier, rnd.draft_logits, rnd.tree_token,
                                         rnd.tree_parent, rnd.mask_bits, O, lse, rnd.accept_len, rnd.accept_path,
                                         rnd.bonus_token)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b), "two runs on the same inputs differ bitwise"


def test_many_row_round_is_bitwise_reproducible():
    """The same for a batch whose passes take the many-row LM head: its per-row kernel appends candidates to a list
    in LDS in whatever order the waves arrive, which must not show in any output."""
    from paper_2406_16858_amd import DraftRound
    cfg = _cfg("repro_many_rows", batch=6, vocab=20011, hidden=512, depth=4, topk=5, n_tree=30, accept="mixed",
               prefix_lo=3, prefix_hi=200, seed=23)
    B = cfg.batch
    W = wl.make_lm_head(cfg, "cuda")
    H = wl.make_hidden_states(cfg, "cuda", scale=5.0)
    plens = wl.make_prefix_lengths(cfg)
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=plens)
    tl, _ = wl.make_target_logits(cfg, "cuda")
    ua, ub = wl.make_uniforms(cfg, "cuda")
    root = (torch.arange(B, dtype=torch.int32) + 5).cuda()
    plen = torch.tensor(plens, dtype=torch.int32, device="cuda")
    mode = torch.tensor([b % 2 for b in range(B)], dtype=torch.int32, device="cuda")
    outs = []
    for rep in range(3):
        rnd = DraftRound(B, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, cfg.n_tree, cfg.dtype, cfg.n_q_heads,
                         cfg.n_kv_heads, cfg.head_dim, total_prefix=sum(plens), keep_draft_logits=True)
        rnd.workspace.fill_(rep * 41 + 3)
        rnd.expand_all(H, W)
        rnd.rerank(root, plen)
        O = torch.empty_like(Q)
        rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, None)
        rnd.accept(mode, tl, torch.full((B,), 0.8, device="cuda"), ua, ub)
        torch.cuda.synchronize()
        outs.append([t.clone() for t in (rnd.cand_token, rnd.cand_score, rnd.cand_parent, rnd.frontier, rnd.draft_logits,
                                         rnd.tree_token, rnd.tree_parent, rnd.mask_bits, O, rnd.accept_len, rnd.accept_path,
                                         rnd.bonus_token)])
    for other in outs[1:]:
        for a, b in zip(outs[0], other):
            assert torch.equal(a, b), "two runs on the same inputs differ bitwise"
    assert int(outs[0][0].min()) >= 0 and int(outs[0][9].min()) >= 0


def test_errors_enqueue_nothing():
    from paper_2406_16858_amd import DraftRound, Eagle2Error, binding as b
    cfg = wl.get_config(1)
    rnd = DraftRound(1, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, cfg.n_tree, cfg.dtype, cfg.n_q_heads,
                     cfg.n_kv_heads, cfg.head_dim, total_prefix=128)
    W = wl.make_lm_head(cfg, "cuda")
    H = wl.make_hidden_states(cfg, "cuda")
    before = rnd.cand_token.clone()
    small = torch.empty(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(Eagle2Error, match="workspace"):
        b.eagle2_expand(rnd.cfg, 0, H[:, 0], W, rnd.cand_token, rnd.cand_score, rnd.cand_parent, rnd.frontier, None, small)
    with pytest.raises(Eagle2Error, match="pass index"):
        b.eagle2_expand(rnd.cfg, cfg.depth, H[:, 0], W, rnd.cand_token, rnd.cand_score, rnd.cand_parent, rnd.frontier,
                        None, rnd.workspace)
    with pytest.raises(Eagle2Error, match="aligned"):
        b.eagle2_expand(rnd.cfg, 0, H.view(-1)[1:1 + cfg.hidden], W, rnd.cand_token, rnd.cand_score, rnd.cand_parent,
                        rnd.frontier, None, rnd.workspace)
    torch.cuda.synchronize()
    assert torch.equal(before, rnd.cand_token)
    lib = b.load_library()
    assert lib.eagle2_kernel_timing_read(7, ctypes.byref(ctypes.c_double()), ctypes.byref(ctypes.c_int32())) == -1


@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_partly_filled_kv_regions(dtype):
    """prefix_len selects the filled part of each sequence's region: empty, partial, exactly full,
    larger than the region (clamped) and negative (treated as empty) all equal the oracle on the
    truncated prefix, and rows beyond the filled part have no influence."""
    from oracle import eagle2_oracle as orc
    from paper_2406_16858_amd import DraftRound
    from tests import parity_utils as pu
    cfg = _cfg("kv_regions", dtype=dtype, batch=5, hidden=512 if dtype == "bf16" else 256, n_tree=12, seed=77,
               n_q_heads=4, n_kv_heads=2, head_dim=64)
    B, N = cfg.batch, cfg.n_tree
    region = [150, 150, 150, 150, 150]
    plen = [0, 97, 150, 400, -3]
    want_len = [0, 97, 150, 150, 0]
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    Kp[off[1] + 97: off[2]] = float("nan")             # unfilled rows of sequence 1 hold garbage
    Vp[off[1] + 97: off[2]] = float("nan")
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, N, cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     total_prefix=sum(region))
    # a chain tree: row i sees rows 0..i
    mask = np.tril(np.ones((N, N), dtype=bool))
    bits = np.array([[sum(1 << j for j in range(i + 1))] for i in range(N)], dtype=np.uint64)
    rnd.mask_bits.copy_(torch.from_numpy(np.tile(bits, (B, 1, 1)).view(np.int64)))
    O = torch.full_like(Q, float("nan"))
    lse = torch.full((B, N, cfg.n_q_heads), float("nan"), dtype=torch.float32, device="cuda")
    rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse, prefix_len=torch.tensor(plen, dtype=torch.int32, device="cuda"))
    torch.cuda.synchronize()
    assert not torch.isnan(O.float()).any()
    offs = off.cpu().numpy()
    for b in range(B):
        lo = int(offs[b])
        ref, ref_lse = orc.tree_attn(pu.f64(Q[b]), pu.f64(Kp[lo:lo + want_len[b]]), pu.f64(Vp[lo:lo + want_len[b]]),
                                     pu.f64(Kt[b]), pu.f64(Vt[b]), mask)
        e = pu.rel_err(pu.f64(O[b]), ref)
        assert e <= pu.REL_TOL[dtype], f"seq {b} (prefix_len {plen[b]}): rel err {e:.2e}"
        assert np.max(np.abs(pu.f64(lse[b]) - ref_lse)) <= pu.REL_TOL[dtype] * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("fp8", [False, True], ids=["bf16_prefix", "fp8_prefix"])
def test_long_context_prefix_many_chunks(fp8):
    """A 300k-token prefix: more than 64 key chunks per sequence (the combine kernel walks them in
    batches of 64), next to a short sequence in the same launch."""
    from oracle import eagle2_oracle as orc
    from oracle import fp8_kv_oracle as f8
    from paper_2406_16858_amd import DraftRound
    from tests import parity_utils as pu
    cfg = _cfg("long_ctx", batch=2, n_tree=24, n_q_heads=2, n_kv_heads=1, head_dim=128, seed=88)
    B, N = cfg.batch, cfg.n_tree
    region = [300_001, 70]
    Q, Kp, Vp, Kt, Vt, off = wl.make_attention_inputs(cfg, "cuda", prefix_lens=region)
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, cfg.depth, cfg.topk, N, cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     total_prefix=sum(region))
    mask = np.tril(np.ones((N, N), dtype=bool))
    bits = np.array([[sum(1 << j for j in range(i + 1))] for i in range(N)], dtype=np.uint64)
    rnd.mask_bits.copy_(torch.from_numpy(np.tile(bits, (B, 1, 1)).view(np.int64)))
    O = torch.full_like(Q, float("nan"))
    lse = torch.full((B, N, cfg.n_q_heads), float("nan"), dtype=torch.float32, device="cuda")
    if fp8:
        K8, V8, ks, vs = wl.make_fp8_prefix(Kp, Vp)
        rnd.tree_attn_fp8kv(Q, K8, V8, ks, vs, off, Kt, Vt, O, lse)
        Kd = torch.from_numpy(f8.dequantize(K8.cpu().numpy(), ks.cpu().numpy()))
        Vd = torch.from_numpy(f8.dequantize(V8.cpu().numpy(), vs.cpu().numpy()))
    else:
        rnd.tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse)
        Kd, Vd = Kp, Vp
    torch.cuda.synchronize()
    offs = off.cpu().numpy()
    for b in range(B):
        lo, hi = int(offs[b]), int(offs[b + 1])
        ref, ref_lse = orc.tree_attn(pu.f64(Q[b]), pu.f64(Kd[lo:hi]), pu.f64(Vd[lo:hi]), pu.f64(Kt[b]), pu.f64(Vt[b]), mask)
        e = pu.rel_err(pu.f64(O[b]), ref)
        assert e <= pu.REL_TOL["bf16"], f"seq {b}: rel err {e:.2e}"
        assert np.max(np.abs(pu.f64(lse[b]) - ref_lse)) <= pu.REL_TOL["bf16"] * max(1.0, np.abs(ref_lse).max())


@pytest.mark.parametrize("batch,vocab", [(1, 5003), (20, 5003), (18, 40001)], ids=["few_rows", "many_rows", "many_rows_three_pieces"])
@pytest.mark.parametrize("dtype", ["bf16", "fp32"])
def test_exact_ties_take_the_lower_token_id(batch, vocab, dtype):
    """Rows of W repeated in pairs give logits that tie exactly; hidden states of zero tie every logit.
    Whatever lane, wave or workgroup holds them, equal values must come out lower token id first
    (Section 4.1 leaves the order of equal values open; this build fixes it, as the oracle does)."""
    from paper_2406_16858_amd import DraftRound
    cfg = _cfg("ties", dtype=dtype, batch=batch, vocab=vocab, hidden=512 if dtype == "bf16" else 256, depth=3, topk=5, n_tree=12, seed=17)
    B, D, k, V = cfg.batch, cfg.depth, cfg.topk, cfg.vocab
    W = wl.make_lm_head(cfg, "cuda")
    W[1::2] = W[0:V - 1:2]                             # token 2j+1 repeats token 2j (V is odd: the last token stays single)
    H = wl.make_hidden_states(cfg, "cuda", scale=4.0)
    for zero_h in (False, True):
        if zero_h:
            H = torch.zeros_like(H)
        rnd = DraftRound(B, V, cfg.hidden, D, k, cfg.n_tree, cfg.dtype)
        rnd.expand_all(H, W)
        torch.cuda.synchronize()
        tok = rnd.cand_token.cpu().numpy().reshape(B, -1)
        sc = rnd.cand_score.cpu().numpy().reshape(B, -1)
        par = rnd.cand_parent.cpu().numpy().reshape(B, -1)
        for b in range(B):
            for base in range(0, tok.shape[1], k):     # every expanded row's k children, best first
                t, s, p = tok[b, base:base + k], sc[b, base:base + k], par[b, base:base + k]
                if p[0] < -1 or not np.isfinite(s).all():
                    continue                           # (rows of passes that were not expanded)
                local = s - (sc[b, p[0]] if p[0] >= 0 else 0.0)     # the children's own log-probabilities
                assert np.all(np.diff(local) <= 1e-12), (b, base, local)
                if zero_h:
                    assert list(t) == list(range(k)), (b, base, t)
                    assert np.allclose(local, -np.log(V), atol=1e-5)
                    continue
                chosen = set(int(x) for x in t)
                for i, x in enumerate(t):
                    x = int(x)
                    if x % 2 == 1:                     # a repeated row: its twin comes right before it
                        assert x - 1 in chosen and int(t[i - 1]) == x - 1 and abs(local[i] - local[i - 1]) < 1e-12, (b, base, t, local)
                    elif x + 1 < V and i + 1 < k:      # the twin of an even token ties with it and follows, unless the list ends
                        assert int(t[i + 1]) == x + 1, (b, base, t)
