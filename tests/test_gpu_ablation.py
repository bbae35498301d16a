"""GPU parity of the ablation switches of Section 5.2 (Table 3): expansion ranked by
confidence instead of value, and the draft taken from the expansion phase without the
global re-selection.  Every stage of the round is still checked against the oracle
(attention and acceptance run on the ablated tree)."""
import dataclasses

import numpy as np
import pytest
import torch

import workloads as wl
from tests.parity_utils import FLAG_NO_RERANK, FLAG_RANK_BY_CONFIDENCE, run_and_check_round
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu

FLAGS = [FLAG_RANK_BY_CONFIDENCE, FLAG_NO_RERANK, FLAG_RANK_BY_CONFIDENCE | FLAG_NO_RERANK]
NAMES = ["wo_value", "wo_rerank", "wo_both"]


def _with_tree(cfg, flags):
    """Without reranking the tree is the D*k expanded nodes plus the root."""
    return dataclasses.replace(cfg, n_tree=cfg.depth * cfg.topk + 1) if flags & FLAG_NO_RERANK else cfg


@pytest.mark.parametrize("flags", FLAGS, ids=NAMES)
@pytest.mark.parametrize("base", [wl.get_config(1), _small("abl_batch3", batch=3, accept="mixed", prefix_lo=1, prefix_hi=300, seed=21),
                                  _small("abl_k16", topk=16, depth=3, vocab=2048, n_tree=40, seed=22),
                                  _small("abl_d1", depth=1, n_tree=5, seed=23)],
                         ids=["cfg1", "batch3", "k16", "depth1"])
def test_ablation_small(base, flags):
    cfg = _with_tree(base, flags)
    rep, trees, _ = run_and_check_round(cfg, h_scale=6.0, plant=(cfg.accept == "greedy"), flags=flags)
    if flags & FLAG_NO_RERANK:
        assert all(np.bincount(t.depth).tolist() == [1] + [cfg.topk] * cfg.depth for t in trees)


@pytest.mark.parametrize("flags", FLAGS, ids=NAMES)
def test_ablation_cfg2_paper_shape(flags):
    """LLaMA2-7B shape with the paper's k = 10, D = 6; without reranking the tree has 61 rows."""
    cfg = _with_tree(wl.get_config(2), flags)
    run_and_check_round(cfg, h_scale=6.0, plant=True, flags=flags, attn_heads=[0, 17, 31])


def test_ablation_changes_the_tree():
    """On peaked inputs the switches select different trees than the full method (otherwise
    the tests above would prove nothing)."""
    cfg = _small("abl_diff", seed=31, batch=2)
    _, full, _ = run_and_check_round(cfg, h_scale=6.0, verbose=False)
    _, conf, _ = run_and_check_round(cfg, h_scale=6.0, verbose=False, flags=FLAG_RANK_BY_CONFIDENCE)
    _, flat, _ = run_and_check_round(_with_tree(cfg, FLAG_NO_RERANK), h_scale=6.0, verbose=False, flags=FLAG_NO_RERANK)
    assert any(not np.array_equal(a.token, b.token) for a, b in zip(full, conf))
    assert all(a.token.shape != b.token.shape or not np.array_equal(a.cand, b.cand) for a, b in zip(full, flat))


def test_flag_validation():
    from paper_2406_16858_amd import DraftRound, Eagle2Error
    with pytest.raises(Eagle2Error, match="depth\\*topk"):
        DraftRound(1, 1000, 256, 3, 4, 16, "fp32", flags=FLAG_NO_RERANK)
    with pytest.raises(Eagle2Error, match="unknown bits"):
        DraftRound(1, 1000, 256, 3, 4, 16, "fp32", flags=8)
