"""Guard bands: every output and scratch buffer of every entry point is a view inside a larger
allocation filled with a sentinel; after the kernels have finished the bands on both sides must be
untouched.  (Pre-filling outputs with NaN elsewhere shows entries that were NOT written; this shows
writes that landed OUTSIDE a buffer.)  A pure host-side check of completed kernels, on the tiny fp32
configuration, a ragged multi-sequence shape and the largest tree (N = 128, k = 16)."""
import math

import numpy as np
import pytest
import torch

import workloads as wl
from tests import parity_utils as pu
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu

PAD = 4096
SENTINEL = 0xC3


class Bands:
    def __init__(self, device="cuda"):
        self.device = device
        self.items = []

    def like(self, name, t: torch.Tensor) -> torch.Tensor:
        """A tensor of t's shape, type and contents that sits between two sentinel bands."""
        n = t.numel() * t.element_size()
        buf = torch.full((PAD + n + PAD,), SENTINEL, dtype=torch.uint8, device=self.device)
        view = buf[PAD:PAD + n].view(t.dtype).view(t.shape)
        view.copy_(t)
        assert view.data_ptr() % 16 == 0 and view.is_contiguous()
        self.items.append((name, buf, n))
        return view

    def check(self, where):
        torch.cuda.synchronize()
        for name, buf, n in self.items:
            lo, hi = buf[:PAD], buf[PAD + n:]
            assert bool(torch.all(lo == SENTINEL)), f"{where}: bytes BEFORE {name} were overwritten"
            assert bool(torch.all(hi == SENTINEL)), f"{where}: bytes AFTER {name} were overwritten " \
                                                    f"(first at +{int(torch.nonzero(hi != SENTINEL)[0])})"


ROUND_ARRAYS = ("cand_token", "cand_score", "cand_parent", "frontier", "draft_logits", "tree_token", "tree_parent",
                "tree_depth", "tree_cand", "position_ids", "mask_bits", "accept_len", "accept_path", "bonus_token",
                "workspace")


def _guarded_round_factory(bands):
    from paper_2406_16858_amd import DraftRound

    def make(*a, **kw):
        rnd = DraftRound(*a, **kw)
        for name in ROUND_ARRAYS:
            t = getattr(rnd, name)
            if t is not None:
                setattr(rnd, name, bands.like(name, t))
        real_attn = rnd.tree_attn

        def tree_attn(Q, Kp, Vp, off, Kt, Vt, O, lse=None, prefix_len=None):
            # the harness allocates O and lse itself: run on banded copies and hand the results back
            Og = bands.like("O", O)
            lg = bands.like("lse", lse) if lse is not None else None
            real_attn(Q, Kp, Vp, off, Kt, Vt, Og, lg, prefix_len=prefix_len)
            torch.cuda.synchronize()
            O.copy_(Og)
            if lse is not None:
                lse.copy_(lg)

        rnd.tree_attn = tree_attn
        return rnd

    return make


CASES = [
    (wl.get_config(1), 8.0),
    (_small("bands_ragged", batch=3, vocab=5003, accept="mixed", prefix_lo=1, prefix_hi=700, n_tree=23, seed=91), 6.0),
    (_small("bands_max_tree", topk=16, depth=8, n_tree=128, vocab=3000, accept="sample", prefix_lo=130, prefix_hi=130,
            seed=92), 6.0),
    (_small("bands_many_rows", batch=20, vocab=4099, depth=3, topk=10, n_tree=30, accept="mixed", prefix_lo=0,
            prefix_hi=300, seed=93), 6.0),
]


@pytest.mark.parametrize("cfg,scale", CASES, ids=[c.name for c, _ in CASES])
def test_round_writes_stay_inside_their_buffers(cfg, scale):
    bands = Bands()
    pu.run_and_check_round(cfg, h_scale=scale, plant=True, round_factory=_guarded_round_factory(bands), verbose=False)
    bands.check(cfg.name)
    assert len(bands.items) >= len(ROUND_ARRAYS)


def test_commit_writes_stay_inside_their_buffers():
    from paper_2406_16858_amd import DraftRound
    dev, B, N, D, Hkv, dh, Hd = "cuda", 3, 24, 4, 2, 64, 512
    bands = Bands()
    rnd = DraftRound(B, 5003, Hd, D, 5, N, "bf16", 8, Hkv, dh, total_prefix=3 * 50)
    g = torch.Generator().manual_seed(9)
    Kt = torch.randn((2, B, N, Hkv, dh), generator=g).to(torch.bfloat16).to(dev)
    Vt = torch.randn((2, B, N, Hkv, dh), generator=g).to(torch.bfloat16).to(dev)
    Kc = bands.like("K_cache", torch.zeros((2, 150, Hkv, dh), dtype=torch.bfloat16, device=dev))
    Vc = bands.like("V_cache", torch.zeros((2, 150, Hkv, dh), dtype=torch.bfloat16, device=dev))
    off = torch.tensor([0, 50, 100, 150], dtype=torch.int64, device=dev)
    plen = bands.like("prefix_len", torch.tensor([10, 47, 49], dtype=torch.int32, device=dev))   # regions 1 and 2 overflow
    rnd.accept_len.copy_(torch.tensor([4, 4, 2], dtype=torch.int32))
    rnd.accept_path.copy_(torch.tensor([[0, 2, 5, 9, 23], [0, 1, 3, 8, 20], [0, 4, 7, -1, -1]], dtype=torch.int32))
    rnd.bonus_token.copy_(torch.tensor([5, 6, 7], dtype=torch.int32))
    rnd.commit_kv(off, plen, Kt, Vt, Kc, Vc, n_layers=2, tree_layer_stride=Kt[0].numel(), cache_layer_stride=Kc[0].numel())
    hid = torch.randn((B, N, Hd), generator=g).to(torch.bfloat16).to(dev)
    nxt = bands.like("next_hidden", torch.zeros((B, Hd), dtype=torch.bfloat16, device=dev))
    out = bands.like("out_tokens", torch.zeros((B, D + 1), dtype=torch.int32, device=dev))
    root = bands.like("root_token", torch.zeros((B,), dtype=torch.int32, device=dev))
    rnd.commit_round(out, root, plen, hid, nxt)
    bands.check("commit")
    # rows that would fall beyond a region are dropped, not written into the next region
    assert torch.all(Kc[:, 50:50 + 47] == 0) and torch.all(Kc[:, 100:100 + 49] == 0)
    assert torch.equal(Kc[1, 97], Kt[1, 1, 0]) and torch.equal(Kc[1, 99], Kt[1, 1, 3]) and torch.equal(Kc[0, 149], Kt[0, 2, 0])


def test_draft_forward_writes_stay_inside_their_buffers():
    from paper_2406_16858_amd import DraftModel, DraftRound
    dev = "cuda"
    cfg = _small("bands_draft", batch=2, vocab=2048, hidden=512, depth=3, topk=5, n_tree=12, prefix_lo=3, prefix_hi=90, seed=94)
    dl = wl.DraftLayerConfig(8, 2, 64, 1024, 1e-5, 10000.0)
    B, D = cfg.batch, cfg.depth
    plens = wl.make_prefix_lengths(cfg)
    bands = Bands()
    rnd = DraftRound(B, cfg.vocab, cfg.hidden, D, cfg.topk, cfg.n_tree, cfg.dtype, device=dev)
    for name in ("cand_token", "cand_score", "cand_parent", "frontier", "workspace"):
        setattr(rnd, name, bands.like(name, getattr(rnd, name)))
    dm = DraftModel(rnd, wl.make_draft_weights(cfg, dl, dev), dl.n_q_heads, dl.n_kv_heads, dl.head_dim, dl.intermediate,
                    dl.eps, dl.rope_theta, sum(plens))
    for name in ("feature", "K", "V", "mask", "workspace"):
        setattr(dm, name, bands.like("draft_" + name, getattr(dm, name)))
    acfg = wl.RoundConfig(**{**cfg.__dict__, "n_q_heads": dl.n_q_heads, "n_kv_heads": dl.n_kv_heads, "head_dim": dl.head_dim})
    _, Kp, Vp, _, _, off = wl.make_attention_inputs(acfg, dev, layer=3, prefix_lens=plens)
    plen_t = torch.tensor(plens, dtype=torch.int32, device=dev)
    root = (torch.arange(B, dtype=torch.int32) * 5 + 3).to(dev)
    root_feat = wl.SeededStream(cfg, 40, 0, dev).normal((B, cfg.hidden), 1.0, torch.bfloat16)
    W = wl.make_lm_head(cfg, dev)
    for d in range(D):
        dm.forward(d, root, root_feat, plen_t, Kp, Vp, off)
        dm.expand(d, W)
    bands.check("draft forward")
    assert math.isfinite(float(dm.feature.float().abs().max()))
