"""GPU parity on shapes drawn from a seeded generator: every supported dimension varies at once
(vocabulary with ragged tails, hidden size, depth, children per node, tree size, batch, head
layout, ragged prefixes, accept mode, temperature), each round checked stage by stage against
the oracle like the hand-picked cases."""
import numpy as np
import pytest

import workloads as wl
from tests.parity_utils import run_and_check_round

pytestmark = pytest.mark.gpu


def _draw(i):
    rng = np.random.default_rng(9000 + i)
    dtype = "fp32" if rng.random() < 0.3 else "bf16"
    unit = 256 if dtype == "fp32" else 512                   # a row of W is a multiple of 1 KiB
    hidden = unit * int(rng.integers(1, 4))
    k = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 10, 13, 16]))
    D = int(rng.integers(1, 7))
    C = k + (D - 1) * k * k
    n_tree = int(rng.integers(2, min(128, C + 1) + 1))
    vocab = int(rng.integers(max(16, k), 7000))
    batch = int(rng.choice([1, 1, 2, 3, 5, 9, 18]))          # 18 * k > 16 rows for most k: the many-row LM head
    if batch * k > 64:
        vocab = min(vocab, 3000)                             # keeps the oracle's work small
    dh = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 4]))
    grp = int(rng.choice([1, 2, 4, 8]))
    p_hi = int(rng.choice([0, 1, 63, 64, 65, 200, 700, 2500]))
    p_lo = int(rng.integers(0, p_hi + 1))
    accept = str(rng.choice(["greedy", "sample", "mixed"]))
    return wl.RoundConfig(name=f"random{i}", index=0, dtype=dtype, batch=batch, vocab=vocab, hidden=hidden, depth=D, topk=k,
                          n_tree=n_tree, n_q_heads=hkv * grp, n_kv_heads=hkv, head_dim=dh, prefix_lo=p_lo, prefix_hi=p_hi,
                          n_layers=1, w_std=0.05, accept=accept, temperature=float(rng.choice([1.0, 0.7, 1.5])), seed=500 + i)


CASES = [_draw(i) for i in range(24)]


@pytest.mark.parametrize("cfg", CASES, ids=[f"{c.name}_{c.dtype}_V{c.vocab}_h{c.hidden}_D{c.depth}_k{c.topk}_N{c.n_tree}_B{c.batch}_"
                                            f"{c.n_q_heads}x{c.n_kv_heads}x{c.head_dim}_P{c.prefix_lo}-{c.prefix_hi}_{c.accept}" for c in CASES])
def test_random_shape(cfg):
    run_and_check_round(cfg, h_scale=5.0, plant=(cfg.accept == "greedy"), verbose=False)


def _draw_many_rows(i):
    """More than 16 frontier rows per pass and vocabularies of one to five 16384-entry pieces: the many-row LM head and
    its per-row kernel at every list size."""
    rng = np.random.default_rng(77000 + i)
    dtype = "fp32" if rng.random() < 0.25 else "bf16"
    hidden = (256 if dtype == "fp32" else 512) * int(rng.integers(1, 3))
    k = int(rng.choice([2, 3, 4, 5, 8, 10, 13, 16]))
    batch = int(rng.choice([2, 3, 5, 9, 18]))
    while batch * k <= 16:
        batch += 3
    D = int(rng.integers(2, 5))
    C = k + (D - 1) * k * k
    n_tree = int(rng.integers(2, min(128, C + 1) + 1))
    vocab = int(rng.integers(3000, 70000))
    if batch * k > 100:
        vocab = min(vocab, 30000)                            # keeps the oracle's work small
    hkv = int(rng.choice([1, 2]))
    grp = int(rng.choice([1, 2, 4]))
    p_hi = int(rng.choice([0, 5, 64, 200]))
    p_lo = int(rng.integers(0, p_hi + 1))
    accept = str(rng.choice(["greedy", "sample", "mixed"]))
    return wl.RoundConfig(name=f"manyrows{i}", index=0, dtype=dtype, batch=batch, vocab=vocab, hidden=hidden, depth=D, topk=k,
                          n_tree=n_tree, n_q_heads=hkv * grp, n_kv_heads=hkv, head_dim=64, prefix_lo=p_lo, prefix_hi=p_hi,
                          n_layers=1, w_std=0.05, accept=accept, temperature=float(rng.choice([1.0, 0.7, 1.5])), seed=900 + i)


MANY = [_draw_many_rows(i) for i in range(16)]


@pytest.mark.parametrize("i,cfg", list(enumerate(MANY)), ids=[f"{c.name}_{c.dtype}_V{c.vocab}_h{c.hidden}_D{c.depth}_k{c.topk}_N{c.n_tree}_B{c.batch}_{c.accept}"
                                                              for c in MANY])
def test_random_many_row_shape(i, cfg):
    run_and_check_round(cfg, h_scale=(1.0, 5.0)[i % 2], plant=(cfg.accept == "greedy"), verbose=False)
