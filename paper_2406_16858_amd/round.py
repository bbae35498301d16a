"""Device buffers of one draft-plus-verify round and the order of the C-ABI calls.

DraftRound owns the caller-side arrays the C ABI works on (candidate arrays,
frontier, flattened tree, mask, workspace) as torch device tensors and issues the
calls in the order of the method: D x expand (Section 4.1), rerank (Section 4.2),
tree attention once per layer, accept (Sections 2.1/2.2).  It computes nothing
itself.
"""
from __future__ import annotations

from typing import Optional

import torch

from . import binding as _b


class DraftRound:
    def __init__(self, batch: int, vocab: int, hidden: int, depth: int, topk: int, n_tree: int, dtype: str,
                 n_q_heads: int = 0, n_kv_heads: int = 0, head_dim: int = 0, total_prefix: int = 0,
                 keep_draft_logits: bool = False, device="cuda", flags: int = 0,
                 static_tree: Optional[torch.Tensor] = None):
        """static_tree: [n_tree - 1] int32 device tensor of candidate ids (with FLAG_STATIC_TREE; the caller
        also fills self.frontier with the candidate ids each pass expands)."""
        self.device = torch.device(device)
        self.static_tree = static_tree                 # kept alive: the struct holds a raw pointer
        st_ptr = None
        if static_tree is not None:
            if not static_tree.is_cuda or static_tree.dtype != torch.int32 or static_tree.numel() != n_tree - 1:
                raise _b.Eagle2Error("static_tree must be an int32 device tensor of n_tree - 1 candidate ids")
            st_ptr = static_tree.data_ptr()
        self.cfg = _b.RoundCfg(batch, vocab, hidden, depth, topk, n_tree,
                               _b.DTYPE_F32 if dtype == "fp32" else _b.DTYPE_BF16, flags, st_ptr)
        self.attn: Optional[_b.AttnCfg] = None
        if n_q_heads:
            self.attn = _b.AttnCfg(n_q_heads, n_kv_heads, head_dim, 0.0, total_prefix)
        B, C, D, k, N = batch, self.cfg.n_cand, depth, topk, n_tree
        dev = self.device
        i32 = torch.int32
        self.cand_token = torch.full((B, C), -1, dtype=i32, device=dev)
        self.cand_score = torch.full((B, C), float("-inf"), dtype=torch.float64, device=dev)
        self.cand_parent = torch.full((B, C), -1, dtype=i32, device=dev)
        self.frontier = torch.full((B, D, k), -1, dtype=i32, device=dev)
        self.draft_logits = (torch.zeros((B, self.cfg.n_draft_rows, vocab), dtype=torch.float32, device=dev)
                             if keep_draft_logits else None)
        self.tree_token = torch.zeros((B, N), dtype=i32, device=dev)
        self.tree_parent = torch.zeros((B, N), dtype=i32, device=dev)
        self.tree_depth = torch.zeros((B, N), dtype=i32, device=dev)
        self.tree_cand = torch.zeros((B, N), dtype=i32, device=dev)
        self.position_ids = torch.zeros((B, N), dtype=i32, device=dev)
        self.mask_bits = torch.zeros((B, N, (N + 63) // 64), dtype=torch.int64, device=dev)
        self.accept_len = torch.zeros((B,), dtype=i32, device=dev)
        self.accept_path = torch.zeros((B, D + 1), dtype=i32, device=dev)
        self.bonus_token = torch.zeros((B,), dtype=i32, device=dev)
        nbytes = _b.eagle2_workspace_bytes(self.cfg, self.attn)
        if nbytes == 0:
            raise _b.Eagle2Error("unsupported shape: " + _b.load_library().eagle2_last_error().decode())
        self.workspace = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=dev)

    # -- Section 4.1 ---------------------------------------------------------------
    def expand(self, d: int, H: torch.Tensor, W: torch.Tensor, h_seq_stride: int = 0):
        """H: [B, F_d, Hd] (or a view whose sequences are h_seq_stride elements apart)."""
        _b.eagle2_expand(self.cfg, d, H, W, self.cand_token, self.cand_score, self.cand_parent, self.frontier,
                         self.draft_logits, self.workspace, h_seq_stride)

    def expand_all(self, H_all: torch.Tensor, W: torch.Tensor):
        """H_all: [B, D, k, Hd]: hidden state per (sequence, pass, frontier slot)."""
        B, D, k, Hd = H_all.shape
        for d in range(D):
            self.expand(d, H_all[:, d], W, h_seq_stride=D * k * Hd)

    # -- Section 4.2 ---------------------------------------------------------------
    def rerank(self, root_token: torch.Tensor, prefix_len: torch.Tensor):
        _b.eagle2_rerank(self.cfg, self.cand_token, self.cand_score, self.cand_parent, self.frontier, root_token, prefix_len,
                         self.tree_token, self.tree_parent, self.tree_depth, self.tree_cand, self.position_ids,
                         self.mask_bits, self.workspace)

    def tree_attn(self, Q, K_prefix, V_prefix, kv_offsets, K_tree, V_tree, O, lse=None, prefix_len=None):
        _b.eagle2_tree_attn(self.cfg, self.attn, Q, K_prefix, V_prefix, kv_offsets, K_tree, V_tree, self.mask_bits,
                            O, lse, self.workspace, prefix_len=prefix_len)

    def tree_attn_fp8kv(self, Q, K_prefix8, V_prefix8, k_scale, v_scale, kv_offsets, K_tree, V_tree, O, lse=None, prefix_len=None):
        """Same with the prefix keys/values stored as 8-bit E4M3 codes (uint8) and one float scale per KV head."""
        _b.eagle2_tree_attn_fp8kv(self.cfg, self.attn, Q, K_prefix8, V_prefix8, k_scale, v_scale, kv_offsets, K_tree, V_tree,
                                  self.mask_bits, O, lse, self.workspace, prefix_len=prefix_len)

    # -- Sections 2.1 / 2.2 -----------------------------------------------------------
    def accept(self, mode, target_logits, temperature=None, u_accept=None, u_bonus=None):
        _b.eagle2_accept(self.cfg, mode, target_logits, self.draft_logits, temperature, u_accept, u_bonus,
                         self.tree_token, self.tree_parent, self.tree_cand, self.accept_len, self.accept_path,
                         self.bonus_token, self.workspace)

    # -- Section 2.1: what the round leaves behind ----------------------------------------
    def commit_kv(self, kv_offsets, prefix_len, K_tree, V_tree, K_cache, V_cache, n_layers: int = 1,
                  tree_layer_stride: int = 0, cache_layer_stride: int = 0):
        _b.eagle2_commit_kv(self.cfg, self.attn, n_layers, self.accept_len, self.accept_path, kv_offsets, prefix_len,
                            K_tree, V_tree, tree_layer_stride, K_cache, V_cache, cache_layer_stride)

    def commit_kv_fp8(self, kv_offsets, prefix_len, K_tree, V_tree, K_cache8, V_cache8, k_scale, v_scale, n_layers: int = 1,
                      tree_layer_stride: int = 0, cache_layer_stride: int = 0):
        """commit_kv into a cache of 8-bit codes; k_scale/v_scale are [n_layers, Hkv] float32."""
        _b.eagle2_commit_kv_fp8(self.cfg, self.attn, n_layers, self.accept_len, self.accept_path, kv_offsets, prefix_len,
                                K_tree, V_tree, tree_layer_stride, K_cache8, V_cache8, cache_layer_stride, k_scale, v_scale)

    def commit_round(self, out_tokens, root_token, prefix_len, target_hidden=None, next_hidden=None):
        _b.eagle2_commit_round(self.cfg, self.accept_len, self.accept_path, self.tree_token, self.bonus_token,
                               target_hidden, out_tokens, root_token, prefix_len, next_hidden)


class DraftModel:
    """Weights, draft-tree arrays and workspace of the draft model's forward (Section 2.2, drafting
    stage) for one DraftRound.  forward(d) computes the features of pass d's rows; expand(d)
    then reads them in place."""

    def __init__(self, rnd: DraftRound, tensors: dict, n_q_heads: int, n_kv_heads: int, head_dim: int, intermediate: int,
                 eps: float, rope_theta: float, total_prefix: int):
        self.rnd = rnd
        cfg = rnd.cfg
        self.dcfg = _b.DraftCfg(n_q_heads, n_kv_heads, head_dim, intermediate, eps, rope_theta)
        self.tensors = tensors                         # kept alive: the struct holds raw pointers
        self.weights = _b.draft_weights(cfg, tensors)
        self.total_prefix = total_prefix
        B, Rd, dev = cfg.batch, max(cfg.n_draft_rows, 2), rnd.device
        el = torch.float32 if cfg.dtype == _b.DTYPE_F32 else torch.bfloat16
        self.rows = Rd
        self.feature = torch.zeros((B, Rd, cfg.hidden), dtype=el, device=dev)
        self.K = torch.zeros((B, Rd, n_kv_heads, head_dim), dtype=el, device=dev)
        self.V = torch.zeros_like(self.K)
        self.mask = torch.zeros((B, Rd, (Rd + 63) // 64), dtype=torch.int64, device=dev)
        nbytes = _b.eagle2_draft_workspace_bytes(cfg, self.dcfg, total_prefix)
        if nbytes == 0:
            raise _b.Eagle2Error("unsupported draft shape: " + _b.load_library().eagle2_last_error().decode())
        self.workspace = torch.empty((nbytes + 255) // 256 * 256, dtype=torch.uint8, device=dev)

    def forward(self, d: int, root_token, root_feature, prefix_len, K_prefix, V_prefix, kv_offsets):
        r = self.rnd
        _b.eagle2_draft_forward(r.cfg, self.dcfg, self.weights, d, r.cand_token, r.cand_parent, r.frontier, root_token,
                                root_feature, prefix_len, K_prefix, V_prefix, kv_offsets, self.total_prefix,
                                self.feature, self.K, self.V, self.mask, self.workspace)

    def expand(self, d: int, W: torch.Tensor):
        """The LM-head pass of layer d on the features just computed (read in place)."""
        k = self.rnd.cfg.topk
        row_base = 0 if d == 0 else 1 + (d - 1) * k
        self.rnd.expand(d, self.feature[:, row_base:], W, h_seq_stride=self.rows * self.rnd.cfg.hidden)
