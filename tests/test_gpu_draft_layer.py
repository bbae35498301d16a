"""GPU parity of the draft model's forward (eagle2_draft_forward) interleaved with the expansion
passes it feeds: per pass the new rows' features, rotary keys, values and ancestor masks are
compared with the oracle, which is fed the GPU's own (rounded) features of the earlier passes, so
rounding does not accumulate across passes; the expansion pass that reads the features in place
is then checked in lock-step as everywhere else."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import draft_layer_oracle as dlo
from oracle import eagle2_oracle as orc
from tests import parity_utils as pu
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu

# same bars as the rest of the path (activations are rounded to bf16 at five points of the layer;
# measured 9e-3 for bf16, 3e-6 for float32)
FEATURE_TOL = pu.REL_TOL


def _run(cfg, dl, verbose=True):
    from paper_2406_16858_amd import DraftModel, DraftRound
    dev = "cuda"
    B, D, k, V, Hd = cfg.batch, cfg.depth, cfg.topk, cfg.vocab, cfg.hidden
    plens = wl.make_prefix_lengths(cfg)
    rnd = DraftRound(B, V, Hd, D, k, cfg.n_tree, cfg.dtype, device=dev)
    tens = wl.make_draft_weights(cfg, dl, dev)
    dm = DraftModel(rnd, tens, dl.n_q_heads, dl.n_kv_heads, dl.head_dim, dl.intermediate, dl.eps, dl.rope_theta, sum(plens))
    w64 = dlo.DraftWeights(**{n: pu.f64(t) for n, t in tens.items()}, n_q_heads=dl.n_q_heads, n_kv_heads=dl.n_kv_heads,
                           head_dim=dl.head_dim, eps=dl.eps, rope_theta=dl.rope_theta)
    el = torch.float32 if cfg.dtype == "fp32" else torch.bfloat16
    # the draft model's own KV prefix (same shape as the attention inputs' prefix, draft head counts)
    acfg = wl.RoundConfig(**{**cfg.__dict__, "n_q_heads": dl.n_q_heads, "n_kv_heads": dl.n_kv_heads, "head_dim": dl.head_dim})
    _, Kp, Vp, _, _, off = wl.make_attention_inputs(acfg, dev, layer=3, prefix_lens=plens)
    plen_t = torch.tensor(plens, dtype=torch.int32, device=dev)
    root = (torch.arange(B, dtype=torch.int32) * 5 + 3).to(dev)
    root_feat = wl.SeededStream(cfg, 40, 0, dev).normal((B, Hd), 1.0, el)
    W = wl.make_lm_head(cfg, dev)
    W64 = pu.f64(W)
    states = [orc.DraftState(D, k) for _ in range(B)]
    rep = pu.Report()
    Rd = dm.rows
    Kt_ref = [np.zeros((Rd, dl.n_kv_heads, dl.head_dim)) for _ in range(B)]
    Vt_ref = [np.zeros((Rd, dl.n_kv_heads, dl.head_dim)) for _ in range(B)]
    mask_ref = np.zeros((B, Rd, Rd), dtype=bool)
    offs = off.cpu().numpy()
    tol, worst = FEATURE_TOL[cfg.dtype], 0.0
    for d in range(D):
        F = 1 if d == 0 else k
        feat_before = pu.f64(dm.feature)                   # the GPU's features of earlier passes
        dm.forward(d, root, root_feat, plen_t, Kp, Vp, off)
        torch.cuda.synchronize()
        feat = pu.f64(dm.feature)
        gK, gV = pu.f64(dm.K), pu.f64(dm.V)
        gmask = dm.mask.cpu().numpy().view(np.uint64)
        for b in range(B):
            st = states[b]
            rows = [orc.draft_row(d, s, k) for s in range(F)]
            if d == 0:
                toks, prev, prow = [int(root[b])], pu.f64(root_feat[b])[None], [-1]
            else:
                cands = [int(c) for c in st.frontier[d]]
                toks = [int(st.token[c]) for c in cands]
                prow = [0 if st.parent[c] < 0 else orc.draft_row(d - 1, list(st.frontier[d - 1]).index(int(st.parent[c])), k)
                        for c in cands]
                prev = feat_before[b, prow]
            for i, r in enumerate(rows):
                mask_ref[b, r] = mask_ref[b, prow[i]] if prow[i] >= 0 else False
                mask_ref[b, r, r] = True
            lo, hi = int(offs[b]), int(offs[b]) + plens[b]
            # the oracle sees the GPU's (rounded) keys and values of earlier rows
            Kt_ref[b][:rows[0]], Vt_ref[b][:rows[0]] = gK[b, :rows[0]], gV[b, :rows[0]]
            want = dlo.draft_layer(w64, toks, prev, np.full(F, plens[b] + d), pu.f64(Kp[lo:hi]), pu.f64(Vp[lo:hi]),
                                   Kt_ref[b], Vt_ref[b], rows, mask_ref[b, rows])
            e = pu.rel_err(feat[b, rows], want)
            ek = pu.rel_err(gK[b, rows], Kt_ref[b][rows])
            ev = pu.rel_err(gV[b, rows], Vt_ref[b][rows])
            worst = max(worst, e, ek, ev)
            assert e <= tol and ek <= tol and ev <= tol, f"seq {b} pass {d}: feature/K/V rel err {e:.2e}/{ek:.2e}/{ev:.2e}"
            for i, r in enumerate(rows):
                bits = sum(1 << j for j in range(Rd) if mask_ref[b, r, j])
                got = sum(int(gmask[b, r, wd]) << (64 * wd) for wd in range(gmask.shape[2]))
                assert got == bits, f"seq {b} pass {d} row {r}: ancestor mask {got:x} != {bits:x}"
        dm.expand(d, W)
        torch.cuda.synchronize()
        row_base = 0 if d == 0 else 1 + (d - 1) * k
        pu.check_expand_pass(rnd, cfg, states, d, feat[:, row_base:row_base + F], W64, rep)
    if verbose:
        print(f"[{cfg.name}] draft layer worst rel err {worst:.2e}; swaps {rep.swaps_topk}/{rep.swaps_frontier}; "
              f"score_err {rep.max_score_err:.2e}", flush=True)
    return worst


@pytest.mark.parametrize("cfg,dl", [
    (_small("draft_bf16", batch=2, vocab=2048, hidden=512, depth=4, topk=5, n_tree=16, prefix_lo=3, prefix_hi=200, seed=51),
     wl.DraftLayerConfig(8, 2, 64, 1024, 1e-5, 10000.0)),
    (_small("draft_fp32", dtype="fp32", batch=1, vocab=777, hidden=256, depth=3, topk=4, n_tree=12, prefix_lo=40, prefix_hi=40, seed=52),
     wl.DraftLayerConfig(4, 4, 64, 768, 1e-6, 500000.0)),
    (_small("draft_bf16_dh128_k10", batch=3, vocab=4096, hidden=1024, depth=3, topk=10, n_tree=20, prefix_lo=0, prefix_hi=90, seed=53),
     wl.DraftLayerConfig(8, 8, 128, 1536, 1e-5, 10000.0)),
    (_small("draft_chain_k1", batch=2, vocab=2048, hidden=512, depth=6, topk=1, n_tree=7, prefix_lo=5, prefix_hi=70, seed=54),
     wl.DraftLayerConfig(8, 2, 64, 1024, 1e-5, 10000.0)),
    (_small("draft_depth1", batch=2, vocab=2048, hidden=512, depth=1, topk=5, n_tree=6, prefix_lo=5, prefix_hi=70, seed=55),
     wl.DraftLayerConfig(8, 8, 64, 512, 1e-5, 10000.0)),
    (_small("draft_k16_rows113", batch=1, vocab=2048, hidden=512, depth=8, topk=16, n_tree=64, prefix_lo=33, prefix_hi=33, seed=56),
     wl.DraftLayerConfig(8, 4, 64, 1024, 1e-5, 10000.0)),
    # more than 16 (and more than 160) rows per pass: the products run through the many-row GEMM
    (_small("draft_rows200", batch=20, vocab=2048, hidden=512, depth=2, topk=10, n_tree=12, prefix_lo=0, prefix_hi=60, seed=57),
     wl.DraftLayerConfig(8, 2, 64, 1024, 1e-5, 10000.0)),
    (_small("draft_rows36_fp32", dtype="fp32", batch=9, vocab=777, hidden=256, depth=3, topk=4, n_tree=10, prefix_lo=5, prefix_hi=30, seed=58),
     wl.DraftLayerConfig(4, 2, 64, 512, 1e-5, 10000.0)),
], ids=["bf16_gqa_dh64", "fp32", "bf16_mha_dh128_rows30", "chain_k1", "depth1_two_row_minimum", "k16_113_draft_rows",
        "rows200_bf16", "rows36_fp32"])
def test_draft_layer_small(cfg, dl):
    _run(cfg, dl)


def test_draft_layer_uneven_k_split():
    """An intermediate size whose rows are an odd number (43) of 256-byte stages, like the 7B models' 11008 (86 stages)."""
    cfg = _small("draft_uneven", batch=1, vocab=2048, hidden=512, depth=3, topk=6, n_tree=12, prefix_lo=9, prefix_hi=9, seed=59)
    _run(cfg, wl.DraftLayerConfig(8, 2, 64, 43 * 128, 1e-5, 10000.0))


def test_draft_layer_llama2_7b_shape():
    _run(wl.get_config(2), wl.DRAFT_LAYERS["llama2_7b"])


def test_draft_layer_llama3_8b_shape():
    """The 8B decoder-layer shape with the headline round configuration (D = 6, k = 10)."""
    cfg = wl.get_config(3)
    _run(cfg, wl.DRAFT_LAYERS["llama3_8b"])


def test_draft_validation():
    from paper_2406_16858_amd import DraftCfg, RoundCfg, eagle2_draft_workspace_bytes, load_library
    cfg = RoundCfg(1, 32000, 4096, 6, 10, 60, 1)
    assert eagle2_draft_workspace_bytes(cfg, DraftCfg(32, 8, 128, 14336, 1e-5, 1e4), 4096) > 0
    assert eagle2_draft_workspace_bytes(cfg, DraftCfg(32, 8, 128, 11008, 1e-5, 1e4), 4096) > 0      # 86 stages of 256 B: uneven split
    assert eagle2_draft_workspace_bytes(cfg, DraftCfg(32, 8, 128, 11000, 1e-5, 1e4), 4096) == 0     # 22000 B is not a multiple of 256
    assert "256" in load_library().eagle2_last_error().decode()
    assert eagle2_draft_workspace_bytes(cfg, DraftCfg(32, 5, 128, 14336, 1e-5, 1e4), 4096) == 0
