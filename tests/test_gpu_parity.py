"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, stage by stage.

Small cases span several 64-row vocab tiles with a ragged tail, several attention tiles
and ragged prefixes; the full-size cases run the five configurations in the launch
configuration the benchmark times.
"""
import numpy as np
import pytest
import torch

import workloads as wl
from tests.parity_utils import run_and_check_round

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2406_16858_amd import load_library
    load_library()


def _small(name, **kw):
    base = dict(name=name, index=0, dtype="bf16", batch=1, vocab=5003, hidden=512, depth=4, topk=5, n_tree=24,
                n_q_heads=8, n_kv_heads=2, head_dim=64, prefix_lo=100, prefix_hi=100, n_layers=1, w_std=0.05,
                accept="greedy", temperature=1.0, seed=1234)
    base.update(kw)
    return wl.RoundConfig(**base)


@pytest.mark.parametrize("scale,plant", [(1.0, False), (8.0, True)])
def test_cfg1_tiny_fp32(scale, plant):
    rep, trees, res = run_and_check_round(wl.get_config(1), h_scale=scale, plant=plant)
    assert rep.swaps_topk == rep.swaps_frontier == rep.swaps_rerank == 0   # fp32 inputs: no near ties expected
    if plant:
        assert res[0].accept_len == int(trees[0].depth.max())


SMALL = [
    _small("ragged_vocab_bf16"),
    _small("ragged_vocab_bf16_sample", accept="sample", seed=77),
    _small("batch3_mixed", batch=3, accept="mixed", prefix_lo=1, prefix_hi=700, seed=5),
    _small("fp32_dh128", dtype="fp32", hidden=256, vocab=777, n_q_heads=4, n_kv_heads=4, head_dim=128, seed=9),
    _small("bf16_dh128_gqa", n_q_heads=16, n_kv_heads=2, head_dim=128, n_tree=40, prefix_lo=300, prefix_hi=300, seed=11),
    _small("k1_chain", topk=1, depth=6, n_tree=7, seed=3),
    _small("k16_n128", topk=16, depth=3, n_tree=128, vocab=2048, seed=4, accept="sample"),
    _small("no_prefix", prefix_lo=0, prefix_hi=0, seed=6),
    _small("temperature_0p7", accept="sample", temperature=0.7, seed=8),
    # more than 16 frontier rows per pass: the logits-then-statistics path of the LM head
    _small("batch20_rows100", batch=20, depth=3, n_tree=16, accept="mixed", prefix_lo=1, prefix_hi=90, seed=12),
    _small("batch41_rows205_fp32", dtype="fp32", batch=41, depth=2, n_tree=12, hidden=256, vocab=4100, n_q_heads=2, n_kv_heads=2,
           prefix_lo=0, prefix_hi=20, seed=13),
    _small("batch5_k16_vocab2048", batch=5, topk=16, depth=2, n_tree=30, vocab=2048, seed=14, accept="sample"),
    # many rows AND more 128-row vocabulary tasks than compute units: every workgroup of the many-row LM head runs
    # several tasks back to back (ring buffers carried across task ends, output stores in mid-stream), ragged last task
    _small("batch3_rows30_vocab100003", batch=3, topk=10, depth=2, n_tree=14, vocab=100003, hidden=512, accept="mixed",
           prefix_lo=0, prefix_hi=50, seed=15),
    _small("batch17_rows170_vocab66000", batch=17, topk=10, depth=2, n_tree=12, vocab=66000, hidden=512, accept="greedy",
           prefix_lo=0, prefix_hi=30, seed=16),
    # the per-row kernel of the many-row path at its three list sizes (k <= 4, <= 10, 16), with vocabularies of one
    # ragged piece, barely sixteen occupied waves, and two pieces per row
    _small("batch2_rows32_k16_vocab20011", batch=2, topk=16, depth=2, n_tree=40, vocab=20011, hidden=512, accept="sample",
           prefix_lo=0, prefix_hi=40, seed=18),
    _small("batch6_rows18_k3_vocab9001_fp32", dtype="fp32", batch=6, topk=3, depth=4, n_tree=20, vocab=9001, hidden=256,
           accept="mixed", prefix_lo=0, prefix_hi=40, seed=19),
    _small("batch2_rows20_k10_vocab4001", batch=2, topk=10, depth=3, n_tree=30, vocab=4001, hidden=512, accept="greedy",
           prefix_lo=5, prefix_hi=60, seed=20),
]


@pytest.mark.parametrize("cfg", SMALL, ids=[c.name for c in SMALL])
@pytest.mark.parametrize("scale", [1.0, 6.0])
def test_small_shapes(cfg, scale):
    run_and_check_round(cfg, h_scale=scale, plant=(scale > 1.0 and cfg.accept != "sample"))


@pytest.mark.parametrize("scale,plant", [(1.0, False), (6.0, True)])
def test_cfg2_llama2_7b(scale, plant):
    run_and_check_round(wl.get_config(2), h_scale=scale, plant=plant)


@pytest.mark.parametrize("scale", [1.0, 6.0])
def test_cfg3_llama3_8b_sampling(scale):
    run_and_check_round(wl.get_config(3), h_scale=scale)


def test_cfg4_llama70b_layer_shape():
    # the round has 80 independent KV layers; parity is checked on two of them, sampled heads
    run_and_check_round(wl.get_config(4), h_scale=6.0, plant=True, layers=(0, 79), attn_heads=range(0, 64, 9))


def test_cfg5_batched_serving():
    run_and_check_round(wl.get_config(5), h_scale=6.0, plant=True, attn_seqs=[0, 5, 10, 15], attn_heads=[0, 13, 31])


@pytest.mark.parametrize("idx", [6, 7])
def test_other_published_settings(idx):
    """Appendix A: 50 draft tokens at the 13B shape, 48 at the 70B shape."""
    cfg = wl.get_config(idx)
    assert cfg.n_tree == {6: 50, 7: 48}[idx] and cfg.depth == 6 and cfg.topk == 10
    run_and_check_round(cfg, h_scale=6.0, plant=(cfg.accept == "greedy"), attn_heads=range(0, cfg.n_q_heads, 7))
