"""GPU parity of the commit step and of several rounds chained through it: every round is
checked stage by stage against the oracle, the KV cache (all layers, whole buffer), the
emitted tokens, the next root, the prefix lengths and the next draft feature bit-exactly,
and the next round's attention runs over the cache the GPU itself has grown
(pre-allocated regions, prefix_len rows filled)."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from oracle import eagle2_oracle as orc
from tests import parity_utils as pu
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu


def _plant(tl, trees, D, B, rnd_idx):
    """Make the target prefer the tokens along a path so accept lengths vary by sequence and round."""
    for b in range(B):
        tree = trees[b]
        j, chain = int(np.argmax(tree.depth)), []
        while j >= 0:
            chain.append(j)
            j = int(tree.parent[j])
        chain.reverse()
        L = min((b + rnd_idx) % (D + 1), len(chain) - 1)
        for i in range(L):
            row = tl[b, chain[i]]
            row[int(tree.token[chain[i + 1]])] = row.max() + 8.0


@pytest.mark.parametrize("base", [
    _small("commit_bf16", batch=3, accept="mixed", prefix_lo=1, prefix_hi=400, seed=41),
    _small("commit_fp32", dtype="fp32", hidden=256, vocab=777, batch=2, n_q_heads=4, n_kv_heads=4, head_dim=128, seed=42),
    wl.get_config(1),
], ids=["bf16_batch3_mixed", "fp32_dh128", "cfg1"])
def test_rounds_chained_through_commit(base):
    from paper_2406_16858_amd import DraftRound
    dev, n_layers, n_rounds = "cuda", 2, 3
    B, D, k, N, V = base.batch, base.depth, base.topk, base.n_tree, base.vocab
    Hkv, dh = base.n_kv_heads, base.head_dim
    plens0 = wl.make_prefix_lengths(base)
    cap = [p + (4 if b == 0 else n_rounds * (D + 1)) for b, p in enumerate(plens0)]   # sequence 0's region overflows in the last round
    offs = np.concatenate([[0], np.cumsum(cap)]).astype(np.int64)
    total = int(offs[-1])
    el = torch.float32 if base.dtype == "fp32" else torch.bfloat16
    # cache [L, total, Hkv, dh], regions partly filled with the seeded prefix
    Kc = torch.zeros((n_layers, total, Hkv, dh), dtype=el, device=dev)
    Vc = torch.zeros_like(Kc)
    for l in range(n_layers):
        _, Kp, Vp, _, _, off0 = wl.make_attention_inputs(base, dev, layer=l, prefix_lens=plens0)
        off0 = off0.cpu().numpy()
        for b in range(B):
            Kc[l, offs[b]:offs[b] + plens0[b]] = Kp[off0[b]:off0[b + 1]]
            Vc[l, offs[b]:offs[b] + plens0[b]] = Vp[off0[b]:off0[b + 1]]
    Kc_ref, Vc_ref = Kc.cpu().clone(), Vc.cpu().clone()
    off_t = torch.from_numpy(offs).to(dev)
    plen_t = torch.tensor(plens0, dtype=torch.int32, device=dev)
    plen_ref = list(plens0)
    root_t = (torch.arange(B, dtype=torch.int32) * 3 + 7).to(dev)
    root_ref = root_t.cpu().numpy().copy()
    modes_l = {"greedy": [0] * B, "sample": [1] * B, "mixed": [b % 2 for b in range(B)]}[base.accept]
    rnd = DraftRound(B, V, base.hidden, D, k, N, base.dtype, base.n_q_heads, Hkv, dh, total_prefix=total,
                     keep_draft_logits=any(modes_l), device=dev)
    W = wl.make_lm_head(base, dev)
    W64 = pu.f64(W)
    seen_lens = set()
    for r in range(n_rounds):
        cfg = dataclasses.replace(base, seed=base.seed + 100 * (r + 1))
        rep = pu.Report()
        H_all = wl.make_hidden_states(cfg, dev, scale=6.0)
        states, rep = pu.lockstep_expand(rnd, cfg, H_all, W, W64=W64, report=rep)
        rnd.rerank(root_t, plen_t)
        torch.cuda.synchronize()
        trees = pu.check_rerank(rnd, cfg, states, root_ref, np.array(plen_ref), rep)
        # tree K/V of all layers in one tensor; attention checked on layer 0 over the grown cache
        Kt = torch.stack([wl.make_attention_inputs(cfg, dev, layer=l, prefix_lens=[0] * B)[3] for l in range(n_layers)])
        Vt = torch.stack([wl.make_attention_inputs(cfg, dev, layer=l, prefix_lens=[0] * B)[4] for l in range(n_layers)])
        Q = wl.make_attention_inputs(cfg, dev, layer=0, prefix_lens=[0] * B)[0]
        O = torch.full_like(Q, float("nan"))
        lse = torch.full((B, N, cfg.n_q_heads), float("nan"), dtype=torch.float32, device=dev)
        rnd.tree_attn(Q, Kc[0], Vc[0], off_t, Kt[0], Vt[0], O, lse, prefix_len=plen_t)
        torch.cuda.synchronize()
        pu.check_attention(cfg, trees, Q, Kc[0], Vc[0], Kt[0], Vt[0], off_t, O, lse, rep, prefix_lens=plen_ref)
        tl, _ = wl.make_target_logits(cfg, dev)
        _plant(tl, trees, D, B, r)
        ua, ub = wl.make_uniforms(cfg, dev)
        temp = torch.full((B,), cfg.temperature, dtype=torch.float32, device=dev)
        rnd.accept(torch.tensor(modes_l, dtype=torch.int32, device=dev), tl, temp, ua, ub)
        torch.cuda.synchronize()
        results = pu.check_accept(rnd, cfg, trees, modes_l, tl, temp.cpu().numpy(), ua, ub, rep)
        # ---- commit: all layers in one call, then the bookkeeping ----
        hid = wl.SeededStream(cfg, 15, 0, dev).normal((B, N, cfg.hidden), 1.0, el)
        nxt = torch.zeros((B, cfg.hidden), dtype=el, device=dev)
        out_tok = torch.full((B, D + 1), -7, dtype=torch.int32, device=dev)
        rnd.commit_kv(off_t, plen_t, Kt, Vt, Kc, Vc, n_layers=n_layers,
                      tree_layer_stride=Kt[0].numel(), cache_layer_stride=Kc[0].numel())
        rnd.commit_round(out_tok, root_t, plen_t, hid, nxt)
        torch.cuda.synchronize()
        Kt_h, Vt_h, hid_h = Kt.cpu(), Vt.cpu(), hid.cpu()
        for b in range(B):
            res = results[b]
            seen_lens.add(res.accept_len)
            for l in range(n_layers):
                orc.commit_kv(Kc_ref[l], Vc_ref[l], int(offs[b]), int(offs[b + 1]), plen_ref[b], Kt_h[l, b], Vt_h[l, b], res.path)
            out = orc.commit_round(trees[b].token, res.path, res.bonus_token, plen_ref[b], hid_h[b].float().numpy())
            want_tok = out.tokens + [-1] * (D + 1 - len(out.tokens))
            assert out_tok[b].tolist() == want_tok, f"round {r} seq {b}: emitted tokens {out_tok[b].tolist()} != {want_tok}"
            assert int(root_t[b]) == out.root_token and int(plen_t[b]) == out.prefix_len
            assert np.array_equal(nxt[b].float().cpu().numpy(), out.next_hidden), f"round {r} seq {b}: next feature differs"
            plen_ref[b], root_ref[b] = out.prefix_len, out.root_token
        assert torch.equal(Kc.cpu(), Kc_ref) and torch.equal(Vc.cpu(), Vc_ref), f"round {r}: committed cache differs"
        print(f"[{base.name} round {r}] accept_len={[x.accept_len for x in results]} prefix_len={plen_ref} "
              f"attn_rel={rep.max_attn_rel:.2e}", flush=True)
    assert len(seen_lens) > 1, "accept lengths did not vary; the commit test would be degenerate"


def test_commit_validation():
    from paper_2406_16858_amd import DraftRound, Eagle2Error
    rnd = DraftRound(1, 1000, 256, 3, 4, 16, "fp32", 4, 4, 64, total_prefix=64)
    z = torch.zeros(64, 4, 64, device="cuda")
    off = torch.tensor([0, 64], dtype=torch.int64, device="cuda")
    pl = torch.zeros(1, dtype=torch.int32, device="cuda")
    kt = torch.zeros(1, 16, 4, 64, device="cuda")
    with pytest.raises(Eagle2Error, match="n_layers"):
        rnd.commit_kv(off, pl, kt, kt, z, z, n_layers=0)
    with pytest.raises(Eagle2Error, match="smaller than one layer"):
        rnd.commit_kv(off, pl, kt, kt, z, z, n_layers=2, tree_layer_stride=16, cache_layer_stride=16)
    with pytest.raises(Eagle2Error, match="together"):
        rnd.commit_round(torch.zeros(1, 4, dtype=torch.int32, device="cuda"), pl.clone(), pl, z[:1, 0], None)


def test_commit_skips_a_sequence_whose_acceptance_failed():
    """eagle2_accept reports an expired wait as accept_len = -1 (forced here from the host: the kernels
    only read it).  The commit calls must leave that sequence's cache region, root, prefix length and
    next feature untouched and emit no token, while the other sequence is committed as usual."""
    from paper_2406_16858_amd import DraftRound
    dev, B, N, D, Hkv, dh, Hd = "cuda", 2, 16, 3, 4, 64, 512
    rnd = DraftRound(B, 1000, Hd, D, 4, N, "bf16", 4, Hkv, dh, total_prefix=2 * 40)
    g = torch.Generator().manual_seed(5)
    Kt = torch.randn((B, N, Hkv, dh), generator=g).to(torch.bfloat16).to(dev)
    Vt = torch.randn((B, N, Hkv, dh), generator=g).to(torch.bfloat16).to(dev)
    Kc = torch.full((2 * 40, Hkv, dh), 3.0, dtype=torch.bfloat16, device=dev)
    Vc = torch.full_like(Kc, -3.0)
    off = torch.tensor([0, 40, 80], dtype=torch.int64, device=dev)
    plen = torch.tensor([10, 20], dtype=torch.int32, device=dev)
    rnd.accept_len.copy_(torch.tensor([-1, 2], dtype=torch.int32))
    rnd.accept_path.copy_(torch.tensor([[-1, -1, -1, -1], [0, 3, 7, -1]], dtype=torch.int32))
    rnd.bonus_token.copy_(torch.tensor([-1, 55], dtype=torch.int32))
    rnd.tree_token.copy_(torch.arange(B * N, dtype=torch.int32).view(B, N) + 100)
    rnd.commit_kv(off, plen, Kt, Vt, Kc, Vc)
    hid = torch.randn((B, N, Hd), generator=g).to(torch.bfloat16).to(dev)
    nxt = torch.full((B, Hd), 9.0, dtype=torch.bfloat16, device=dev)
    out = torch.full((B, D + 1), -7, dtype=torch.int32, device=dev)
    root = torch.tensor([11, 12], dtype=torch.int32, device=dev)
    rnd.commit_round(out, root, plen, hid, nxt)
    torch.cuda.synchronize()
    assert torch.all(Kc[:40] == 3.0) and torch.all(Vc[:40] == -3.0), "the failed sequence's region was written"
    assert out[0].tolist() == [-1] * (D + 1) and int(root[0]) == 11 and int(plen[0]) == 10 and torch.all(nxt[0] == 9.0)
    for i, row in enumerate([0, 3, 7]):
        assert torch.equal(Kc[40 + 20 + i], Kt[1, row]) and torch.equal(Vc[40 + 20 + i], Vt[1, row])
    assert torch.all(Kc[40 + 23:] == 3.0) and torch.all(Kc[40:40 + 20] == 3.0)
    assert out[1].tolist() == [100 + N + 3, 100 + N + 7, 55, -1] and int(root[1]) == 55 and int(plen[1]) == 23
    assert torch.equal(nxt[1], hid[1, 7])
