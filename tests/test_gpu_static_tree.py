"""GPU parity with a fixed-shape draft tree (Section 2.2, "Differences between EAGLE and EAGLE-2":
the shape is fixed and the drafting phase fills in its positions).  The shape is the caller's: the
expansion passes leave the frontiers alone and the flattening takes the shape's nodes as they are;
attention and acceptance then run on that tree as on any other."""
import dataclasses

import numpy as np
import pytest

from tests.parity_utils import FLAG_STATIC_TREE, run_and_check_round
from tests.test_gpu_parity import _small

pytestmark = pytest.mark.gpu

# (parent position in the list, rank among the parent's children), parents first: a small bushy shape
# that narrows with depth, 25 nodes, at most 5 expanded nodes per layer, depth 4
BUSHY = ([(-1, r) for r in range(4)] +                                            # depth 1: ranks 0-3
         [(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (2, 0), (3, 0)] +               # depth 2
         [(4, 0), (4, 1), (4, 2), (5, 0), (5, 1), (7, 0), (8, 0), (9, 0)] +       # depth 3
         [(11, 0), (11, 1), (12, 0), (14, 0), (16, 0), (18, 0)])                  # depth 4
CHAIN = [(-1, 0), (0, 0), (1, 0), (2, 0)]


@pytest.mark.parametrize("nodes,name", [(BUSHY, "bushy"), (CHAIN, "chain")])
@pytest.mark.parametrize("base", [_small("static_bf16", batch=3, accept="mixed", prefix_lo=1, prefix_hi=300, seed=61),
                                  _small("static_fp32", dtype="fp32", hidden=256, vocab=777, n_q_heads=4, n_kv_heads=4, seed=62)],
                         ids=["bf16_batch3_mixed", "fp32"])
def test_static_tree(base, nodes, name):
    cfg = dataclasses.replace(base, n_tree=len(nodes) + 1)
    rep, trees, _ = run_and_check_round(cfg, h_scale=6.0, plant=(cfg.accept == "greedy"), flags=FLAG_STATIC_TREE, static_nodes=nodes)
    depth = []
    for par, _ in nodes:
        depth.append(1 if par < 0 else depth[par] + 1)
    for t in trees:                                         # the tree has exactly the shape's nodes per depth
        assert np.bincount(t.depth).tolist() == [1] + np.bincount(depth)[1:].tolist()
    assert rep.swaps_frontier == 0 and rep.swaps_rerank == 0


def test_static_tree_validation():
    import torch
    from paper_2406_16858_amd import DraftRound, Eagle2Error
    with pytest.raises(Eagle2Error, match="static_tree"):
        DraftRound(1, 1000, 256, 3, 4, 16, "fp32", flags=FLAG_STATIC_TREE)
    st = torch.zeros(15, dtype=torch.int32, device="cuda")
    with pytest.raises(Eagle2Error, match="excludes"):
        DraftRound(1, 1000, 256, 3, 4, 16, "fp32", flags=FLAG_STATIC_TREE | 1, static_tree=st)
