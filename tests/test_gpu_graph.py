"""A whole round (draft layer + expansion passes, rerank, tree attention, accept, commit) recorded
into a HIP graph and replayed: every entry point only enqueues kernels on the caller's stream (no
allocation, no host synchronisation, no memset nodes), so the round is capturable.  Each replay is
compared with the eager result, with eager work and synchronisations between the replays."""
import pytest
import torch

import workloads as wl
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu


def test_round_replays_from_a_graph():
    from paper_2406_16858_amd import DraftModel, DraftRound
    cfg = _small("graph_round", batch=2, vocab=4096, hidden=512, depth=4, topk=5, n_tree=24, accept="mixed",
                 prefix_lo=40, prefix_hi=300, seed=81)
    dl = wl.DraftLayerConfig(8, 2, 64, 1024, 1e-5, 10000.0)
    dev = "cuda"
    B, D, N = cfg.batch, cfg.depth, cfg.n_tree
    plens = wl.make_prefix_lengths(cfg)
    cap = [p + D + 1 for p in plens]
    offs = torch.zeros(B + 1, dtype=torch.int64)
    offs[1:] = torch.cumsum(torch.tensor(cap), 0)
    total = int(offs[-1])
    off_t = offs.to(dev)
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, D, cfg.topk, N, cfg.dtype, cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim,
                     total_prefix=total, keep_draft_logits=True, device=dev)
    dm = DraftModel(rnd, wl.make_draft_weights(cfg, dl, dev), dl.n_q_heads, dl.n_kv_heads, dl.head_dim, dl.intermediate,
                    dl.eps, dl.rope_theta, total)
    W = wl.make_lm_head(cfg, dev)
    Q, _, _, Kt, Vt, _ = wl.make_attention_inputs(cfg, dev, prefix_lens=[0] * B)
    Kc = torch.randn((total, cfg.n_kv_heads, cfg.head_dim), device=dev).bfloat16()
    Vc = torch.randn_like(Kc)
    dKc = torch.randn((total, dl.n_kv_heads, dl.head_dim), device=dev).bfloat16()
    dVc = torch.randn_like(dKc)
    Kc0, Vc0 = Kc.clone(), Vc.clone()
    O = torch.empty_like(Q)
    tl, _ = wl.make_target_logits(cfg, dev)
    ua, ub = wl.make_uniforms(cfg, dev)
    temp = torch.full((B,), 0.9, device=dev)
    mode = torch.tensor([b % 2 for b in range(B)], dtype=torch.int32, device=dev)
    root0 = torch.tensor([3, 8], dtype=torch.int32, device=dev)
    plen0 = torch.tensor(plens, dtype=torch.int32, device=dev)
    root, plen = root0.clone(), plen0.clone()
    feat = torch.randn((B, cfg.hidden), device=dev).bfloat16()
    hid = torch.randn((B, N, cfg.hidden), device=dev).bfloat16()
    nxt = torch.zeros((B, cfg.hidden), dtype=torch.bfloat16, device=dev)
    out_tok = torch.zeros((B, D + 1), dtype=torch.int32, device=dev)

    def reset():
        root.copy_(root0); plen.copy_(plen0); Kc.copy_(Kc0); Vc.copy_(Vc0)

    def one_round():
        for d in range(D):
            dm.forward(d, root, feat, plen, dKc, dVc, off_t)
            dm.expand(d, W)
        rnd.rerank(root, plen)
        rnd.tree_attn(Q, Kc, Vc, off_t, Kt, Vt, O, None, prefix_len=plen)
        rnd.accept(mode, tl, temp, ua, ub)
        rnd.commit_kv(off_t, plen, Kt, Vt, Kc, Vc)
        rnd.commit_round(out_tok, root, plen, hid, nxt)

    def snapshot():
        return [t.clone() for t in (rnd.tree_token, rnd.mask_bits, rnd.cand_score, O, rnd.accept_len, rnd.accept_path,
                                    rnd.bonus_token, out_tok, root, plen, nxt, Kc, Vc, dm.feature)]

    reset(); one_round(); torch.cuda.synchronize()
    want = snapshot()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        reset(); one_round(); torch.cuda.synchronize()          # warm-up on the capture stream
        reset(); torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            one_round()
    torch.cuda.synchronize()
    for rep in range(3):
        reset()
        rnd.workspace.fill_(rep + 1)                          # eager work between the replays
        dm.workspace.fill_(rep + 7)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(snapshot(), want)):
            assert torch.equal(a, b), f"replay {rep}: output {i} differs from the eager round"
