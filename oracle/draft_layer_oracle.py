"""CPU oracle of the draft model's forward pass between two expansion passes.

TEST INFRASTRUCTURE ONLY (same rules as eagle2_oracle.py: imported by tests, the
smoke check and the benchmark's cpu-baseline leg; shares no code with the HIP path).

Section 2.2 ("Drafting Stage"): the draft model autoregresses at the feature level;
its input at a node is the node's token embedding together with the feature of the
position before it (the token sequence is advanced by one step), its output is the
node's feature, which the target's LM head turns into the next token distribution.
Section 4.1: thanks to tree attention all nodes of the current layer go through the
draft model in one forward pass, each seeing the prefix and its own ancestors.

PARITY UNPINNED BY THE PAPER: the paper does not print the draft network itself.
The reading taken here is the network of the models the paper evaluates: one
LLaMA-style decoder layer (RMSNorm, rotary grouped-query attention, SwiGLU MLP,
residual connections) behind a linear fusion of [token embedding ; previous
feature].  The pins (tests/test_oracle_draft_layer.py) check this implementation
against library routines and against running the same layer causally over a whole
sequence at once; they cannot check that the reading is the authors' network.

Everything is float64 numpy, one sequence at a time, plain loops over heads.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional

import numpy as np


@dataclass
class DraftWeights:
    """All matrices are [out, in] (y = x W^T), as the models store them."""
    embed: np.ndarray      # [V, Hd] token embeddings
    fc: np.ndarray         # [Hd, 2 Hd] fusion of [embedding ; feature]
    g_attn: np.ndarray     # [Hd] RMSNorm gain before attention
    wqkv: np.ndarray       # [(Hq + 2 Hkv) dh, Hd]: query rows, then key rows, then value rows
    wo: np.ndarray         # [Hd, Hq dh]
    g_mlp: np.ndarray      # [Hd] RMSNorm gain before the MLP
    wgu: np.ndarray        # [2 I, Hd]: gate rows, then up rows
    wdown: np.ndarray      # [Hd, I]
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    eps: float = 1e-5
    rope_theta: float = 10000.0


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain over the last axis."""
    x = np.asarray(x, dtype=np.float64)
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * np.asarray(gain, dtype=np.float64)


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split convention: element i < dh/2 is paired
    with element i + dh/2 and the pair is rotated by pos * theta^(-2i/dh).
    x [rows, heads, dh], pos [rows]."""
    x = np.asarray(x, dtype=np.float64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / dh)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * inv_freq[None, :]          # [rows, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def draft_layer(w: DraftWeights, tokens, prev_feature, positions, K_prefix, V_prefix, K_tree, V_tree, rows, mask):
    """Forward of the draft layer for the F rows `rows` (indices into the draft tree
    arrays K_tree/V_tree [R, Hkv, dh], which are updated in place with the new keys
    and values).  tokens [F] are the rows' tokens, prev_feature [F, Hd] the feature of
    each row's parent position, positions [F] the rows' position ids, mask [F, R] bool
    the draft-tree rows each new row may see (itself and its ancestors); every row sees
    the whole prefix K_prefix/V_prefix [P, Hkv, dh].  Returns the rows' features [F, Hd].
    """
    Hq, Hkv, dh = w.n_q_heads, w.n_kv_heads, w.head_dim
    tokens = np.asarray(tokens, dtype=np.int64)
    F = tokens.shape[0]
    x_in = np.concatenate([np.asarray(w.embed, dtype=np.float64)[tokens], np.asarray(prev_feature, dtype=np.float64)], axis=-1)
    x0 = x_in @ np.asarray(w.fc, dtype=np.float64).T                               # [F, Hd]
    n1 = rmsnorm(x0, w.g_attn, w.eps)
    qkv = n1 @ np.asarray(w.wqkv, dtype=np.float64).T
    q = qkv[:, : Hq * dh].reshape(F, Hq, dh)
    k = qkv[:, Hq * dh: (Hq + Hkv) * dh].reshape(F, Hkv, dh)
    v = qkv[:, (Hq + Hkv) * dh:].reshape(F, Hkv, dh)
    q = rope(q, positions, w.rope_theta)
    k = rope(k, positions, w.rope_theta)
    for i, r in enumerate(rows):
        K_tree[r] = k[i]
        V_tree[r] = v[i]
    grp = Hq // Hkv
    scale = 1.0 / np.sqrt(dh)
    attn = np.zeros((F, Hq, dh))
    Kp, Vp = np.asarray(K_prefix, dtype=np.float64), np.asarray(V_prefix, dtype=np.float64)
    for i in range(F):
        vis = np.nonzero(np.asarray(mask[i]))[0]
        for h in range(Hq):
            kh = h // grp
            keys = np.concatenate([Kp[:, kh], np.asarray(K_tree, dtype=np.float64)[vis, kh]], axis=0)
            vals = np.concatenate([Vp[:, kh], np.asarray(V_tree, dtype=np.float64)[vis, kh]], axis=0)
            sc = keys @ q[i, h] * scale
            p = np.exp(sc - sc.max())
            attn[i, h] = (p / p.sum()) @ vals
    h1 = x0 + attn.reshape(F, Hq * dh) @ np.asarray(w.wo, dtype=np.float64).T
    n2 = rmsnorm(h1, w.g_mlp, w.eps)
    gu = n2 @ np.asarray(w.wgu, dtype=np.float64).T
    inter = gu.shape[1] // 2
    act = silu(gu[:, :inter]) * gu[:, inter:]
    return h1 + act @ np.asarray(w.wdown, dtype=np.float64).T
